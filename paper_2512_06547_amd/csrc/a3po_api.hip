// extern "C" boundary: argument validation on the host, workspace carve-up, launches.
#include <cmath>
#include <mutex>

#include "a3po.h"
#include "a3po_common.h"
#include "a3po_launch.h"

using namespace a3po;

// Workspace of the entry point that allocates nothing (a3po_loss_fwd_bwd_noalloc): the loss workspace of
// A3PO_NOALLOC_MAX_TOKENS tokens (per-token records, objective, weights, flags, per-workgroup partials, each rounded up
// to 256 bytes).
constexpr size_t kStaticWsBytes = A3PO_NOALLOC_MAX_TOKENS * (size_t)(16 + 4 + 4 + 1) + 6 * 256 + kLossScratchBytes;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

namespace {

using WsLayout = LossWsLayout;

constexpr int64_t kMaxRows = (int64_t)1 << 40, kMaxStride = (int64_t)1 << 40;

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_logits(const void *logits, int dt, int64_t T, int64_t V, int64_t ld)
{
    if (dt != A3PO_F32 && dt != A3PO_BF16) return A3PO_E_DTYPE;
    // (the bounds on T and ld keep every byte offset T * ld * 4 far inside 64 bits)
    if (T < 0 || V <= 0 || ld < V || V > (int64_t)0x7FFFFFFF || T > kMaxRows || ld > kMaxStride) return A3PO_E_SIZE;
    if (T > 0 && !logits) return A3PO_E_NULL;
    if (!aligned(logits, dt == A3PO_F32 ? 4 : 2)) return A3PO_E_ALIGN;  // element alignment; 16 bytes selects the fast kernels
    return A3PO_OK;
}

// ---- workspace of the entry point that allocates nothing ----------------------------------------------
// One array per GPU, part of the loaded code object and held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per device,
// with that device current, and every launch and copy uses the looked-up pointer.

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, 0 until looked up

// device address of the current device's copy of `scratch` (nullptr on failure)
void *static_workspace()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t a3po_workspace_bytes(int which, int64_t T, int64_t V, int64_t H)
{
    if (which == A3PO_WS_LOSS_FWD_BWD) return loss_ws_layout(T).total;
    if (which == A3PO_WS_FUSED_LMHEAD) return lmhead_workspace_bytes(T);
    if (which == A3PO_WS_FUSED_LMHEAD_LOSS) return lmhead_bwd_workspace_bytes(T, V, H);
    return 0;
}

const char *a3po_strerror(int code)
{
    switch (code) {
        case A3PO_OK: return "success";
        case A3PO_E_NULL: return "a required pointer is NULL";
        case A3PO_E_SIZE: return "invalid size (T < 0, V <= 0, ld < V, or bad group structure)";
        case A3PO_E_DTYPE: return "unsupported dtype";
        case A3PO_E_ALIGN: return "pointer is not sufficiently aligned";
        case A3PO_E_WORKSPACE: return "workspace is missing or too small";
        case A3PO_E_LAUNCH: return "HIP rejected a kernel launch";
        case A3PO_E_VALUE: return "scalar argument out of range";
        default: return "unknown a3po error code";
    }
}

int a3po_token_logprobs(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                        float *logp_out, float *lse_out, void *chosen_logit_out, void *stream)
{
    if (int rc = check_logits(logits, (int)dt, T, V, ld)) return rc;
    if (T == 0) return A3PO_OK;
    if (!chosen || !logp_out) return A3PO_E_NULL;
    const hipError_t e = launch_token_logprobs(logits, (int)dt, T, V, ld, chosen, logp_out, lse_out, chosen_logit_out,
                                               nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_token_logprobs_entropy(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                                const int32_t *chosen, float *logp_out, float *lse_out, void *chosen_logit_out,
                                float *entropy_out, void *stream)
{
    if (int rc = check_logits(logits, (int)dt, T, V, ld)) return rc;
    if (T == 0) return A3PO_OK;
    if (!chosen || !logp_out || !entropy_out) return A3PO_E_NULL;
    const hipError_t e = launch_token_logprobs(logits, (int)dt, T, V, ld, chosen, logp_out, lse_out, chosen_logit_out,
                                               entropy_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_proximal_interp(const float *logp_behav, const float *logp_theta, const int32_t *versions,
                         int32_t current_version, int64_t T, float *logp_prox_out, float *alpha_out, void *stream)
{
    if (T < 0) return A3PO_E_SIZE;
    if (T == 0) return A3PO_OK;
    if (!logp_behav || !logp_theta || !versions || !logp_prox_out) return A3PO_E_NULL;
    const hipError_t e = launch_proximal_interp(logp_behav, logp_theta, versions, current_version, T, logp_prox_out,
                                                alpha_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_grpo_advantages(const float *rewards, int64_t S, int32_t G, float eps_adv, const int32_t *seq_id, int64_t T,
                         float *adv_out, void *stream)
{
    if (T < 0 || S < 0 || G <= 0 || S % G != 0) return A3PO_E_SIZE;
    if (!(eps_adv >= 0.0f)) return A3PO_E_VALUE;
    if (T == 0) return A3PO_OK;
    if (!rewards || !seq_id || !adv_out) return A3PO_E_NULL;
    const hipError_t e =
        launch_grpo_advantages(rewards, S, G, eps_adv, seq_id, T, adv_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_fused_lmhead_logprob(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                              const int32_t *chosen, float *logp_out, float *lse_out, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    // H <= 2^20 keeps the kernel's 32-bit byte offsets inside a 256-row tile (255 * 2 H + 64) far below 2^32
    if (T < 0 || V <= 0 || H <= 0 || H % 64 != 0 || H > (1 << 20) || V > (int64_t)0x7FFFFFFF) return A3PO_E_SIZE;
    if (T == 0) return A3PO_OK;
    if (!hidden || !weight || !chosen || !logp_out) return A3PO_E_NULL;
    if (!aligned(hidden, 16) || !aligned(weight, 16)) return A3PO_E_ALIGN;
    if (!workspace || workspace_bytes < lmhead_workspace_bytes(T)) return A3PO_E_WORKSPACE;
    if (!aligned(workspace, 256)) return A3PO_E_ALIGN;
    const hipError_t e = launch_fused_lmhead_logprob(hidden, weight, T, H, V, chosen, logp_out, lse_out, workspace,
                                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_loss_fwd_bwd_ex(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                         const float *logp_behav, const int32_t *versions, int32_t current_version,
                         const float *advantages, const uint8_t *loss_mask, float clip_eps, float denom,
                         void *dlogits, float *logp_out, float *logp_prox_out, float *loss_out,
                         a3po_stats *stats_out, void *workspace, size_t workspace_bytes, void *stream,
                         const a3po_loss_options *opt)
{
    const a3po_loss_options none = {};
    const a3po_loss_options &o = opt ? *opt : none;
    if (int rc = check_logits(logits, (int)dt, T, V, ld)) return rc;
    // (rows, or gradient bursts of rows too long for the registers, are dealt out through a 32-bit counter)
    if (T > kQueueMaxItems || shard_bwd_queue_items((int)dt, T, V) > kQueueMaxItems) return A3PO_E_SIZE;
    if (!(clip_eps >= 0.0f && clip_eps < 1.0f) || std::isnan(denom)) return A3PO_E_VALUE;
    if (o.prox_mode < A3PO_PROX_INTERP || o.prox_mode > A3PO_PROX_BEHAV || (o.accumulate != 0 && o.accumulate != 1))
        return A3PO_E_VALUE;
    if (!loss_out) return A3PO_E_NULL;
    if (T > 0 && (!dlogits || !chosen || !logp_behav || !advantages || !loss_mask || !logp_out)) return A3PO_E_NULL;
    if (T > 0 && o.prox_mode == A3PO_PROX_INTERP && !versions) return A3PO_E_NULL;
    if (T > 0 && o.prox_mode == A3PO_PROX_GIVEN && !o.logp_prox_in) return A3PO_E_NULL;
    if (!aligned(dlogits, dt == A3PO_F32 ? 4 : 2)) return A3PO_E_ALIGN;
    const WsLayout lay = loss_ws_layout(T);
    if (!workspace || workspace_bytes < lay.total) return A3PO_E_WORKSPACE;
    if (!aligned(workspace, 256)) return A3PO_E_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    LossArgs a;
    a.z = logits;
    a.dz = dlogits;
    a.dt = (int)dt;
    a.T = T;
    a.V = V;
    a.ld = ld;
    a.chosen = chosen;
    a.lb = logp_behav;
    a.versions = versions;
    a.current_version = current_version;
    a.adv = advantages;
    a.mask = loss_mask;
    a.clip_eps = clip_eps;
    a.denom = denom;
    a.logp_out = logp_out;
    a.prox_out = logp_prox_out;
    a.loss_out = loss_out;
    a.stats_out = stats_out;
    a.prox_mode = o.prox_mode;
    a.prox_in = o.logp_prox_in;
    a.ent_out = o.entropy_out;
    a.iw_out = o.iw_out;
    a.clipped_out = o.clipped_out;
    a.denom_dev = o.denom_dev;
    a.accumulate = o.accumulate;
    carve_loss_ws(a, workspace, T);

    if (launch_loss_prep(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (o.event_before_rows && hipEventRecord(static_cast<hipEvent_t>(o.event_before_rows), s) != hipSuccess)
        return A3PO_E_LAUNCH;
    if (launch_loss_rows(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (o.event_after_rows && hipEventRecord(static_cast<hipEvent_t>(o.event_after_rows), s) != hipSuccess)
        return A3PO_E_LAUNCH;
    if (launch_loss_finish(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    return A3PO_OK;
}

int a3po_loss_fwd_bwd(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                      const float *logp_behav, const int32_t *versions, int32_t current_version,
                      const float *advantages, const uint8_t *loss_mask, float clip_eps, float denom, void *dlogits,
                      float *logp_out, float *logp_prox_out, float *loss_out, a3po_stats *stats_out, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return a3po_loss_fwd_bwd_ex(logits, dt, T, V, ld, chosen, logp_behav, versions, current_version, advantages,
                                loss_mask, clip_eps, denom, dlogits, logp_out, logp_prox_out, loss_out, stats_out,
                                workspace, workspace_bytes, stream, nullptr);
}

int a3po_loss_fwd_bwd_noalloc(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                              const int32_t *chosen, const float *logp_behav, const int32_t *versions,
                              int32_t current_version, const float *advantages, const uint8_t *loss_mask,
                              float clip_eps, float denom, void *dlogits, float *logp_out, float *logp_prox_out,
                              float *loss_out, a3po_stats *stats_out, void *stream)
{
    if (T > (int64_t)A3PO_NOALLOC_MAX_TOKENS) return A3PO_E_SIZE;
    static_assert(kStaticWsBytes % 256 == 0, "the carve-up below assumes 256-byte granules");
    if (T > 0 && loss_ws_layout(T).total > kStaticWsBytes) return A3PO_E_SIZE;  // (cannot happen below the token limit)
    void *ws = static_workspace();
    if (!ws) return A3PO_E_LAUNCH;
    // Nothing in the array needs clearing here: the prep kernel rewrites the header, the per-token records and the
    // row-queue counter at the start of every call, and every other field is written before it is read.
    return a3po_loss_fwd_bwd_ex(logits, dt, T, V, ld, chosen, logp_behav, versions, current_version, advantages,
                                loss_mask, clip_eps, denom, dlogits, logp_out, logp_prox_out, loss_out, stats_out, ws,
                                kStaticWsBytes, stream, nullptr);
}

int a3po_count_tokens(const int32_t *chosen, const uint8_t *loss_mask, int64_t T, int64_t V, float *denom_out,
                      int64_t *count_out, void *stream)
{
    if (T < 0 || V <= 0) return A3PO_E_SIZE;
    if (!denom_out || (T > 0 && (!chosen || !loss_mask))) return A3PO_E_NULL;
    const hipError_t e =
        launch_count_tokens(chosen, loss_mask, T, V, denom_out, count_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_histogram(const float *values, const uint8_t *select, int64_t T, const float *edges, int32_t nbins,
                   int32_t accumulate, int64_t *counts_out, void *stream)
{
    if (T < 0 || nbins < 1 || nbins > A3PO_HIST_MAX_BINS) return A3PO_E_SIZE;
    if (accumulate != 0 && accumulate != 1) return A3PO_E_VALUE;
    if (!edges || !counts_out || (T > 0 && !values)) return A3PO_E_NULL;
    const hipError_t e = launch_histogram(values, select, T, edges, nbins, accumulate == 1, counts_out,
                                          static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_plan_microbatches(const int64_t *seq_len, int64_t S, int32_t n_minibatches, int64_t max_tokens,
                           int64_t *micro_first_seq, int32_t *micro_minibatch, int64_t capacity, int64_t *n_micro_out)
{
    if (S < 0 || n_minibatches <= 0 || max_tokens <= 0 || capacity < 0) return A3PO_E_SIZE;
    if (!micro_first_seq || !micro_minibatch || !n_micro_out || (S > 0 && !seq_len)) return A3PO_E_NULL;
    for (int64_t s = 0; s < S; ++s)
        if (seq_len[s] < 0) return A3PO_E_SIZE;
    // first pass counts, second pass writes: nothing is written unless everything fits
    for (int pass = 0; pass < 2; ++pass) {
        int64_t n = 0;
        for (int32_t k = 0; k < n_minibatches; ++k) {
            const int64_t lo = (int64_t)k * S / n_minibatches, hi = (int64_t)(k + 1) * S / n_minibatches;
            int64_t tokens = 0;
            bool open = false;
            for (int64_t s = lo; s < hi; ++s) {
                if (!open || (tokens > 0 && seq_len[s] > 0 && tokens + seq_len[s] > max_tokens)) {
                    if (pass == 1) {
                        micro_first_seq[n] = s;
                        micro_minibatch[n] = k;
                    }
                    ++n;
                    tokens = 0;
                    open = true;
                }
                tokens += seq_len[s];
            }
        }
        if (pass == 0 && n > capacity) return A3PO_E_SIZE;
        if (pass == 1) {
            micro_first_seq[n] = S;
            *n_micro_out = n;
        }
    }
    return A3PO_OK;
}

int a3po_shard_partials(const void *logits_shard, a3po_dtype dt, int64_t T, int64_t Vs, int64_t ld,
                        const int32_t *chosen, int64_t v0, a3po_shard_partial *partial_out, void *stream)
{
    if (int rc = check_logits(logits_shard, (int)dt, T, Vs, ld)) return rc;
    if (v0 < 0 || v0 + Vs > (int64_t)0x7FFFFFFF) return A3PO_E_SIZE;
    if (T == 0) return A3PO_OK;
    if (!chosen || !partial_out) return A3PO_E_NULL;
    if (!aligned(partial_out, 16)) return A3PO_E_ALIGN;
    const hipError_t e = launch_shard_partials(logits_shard, (int)dt, T, Vs, ld, chosen, v0, partial_out, nullptr,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_shard_combine(const a3po_shard_partial *partials, int32_t P, int64_t T, const int32_t *chosen, int64_t V,
                       float *logp_out, float *lse_out, float *entropy_out, void *stream)
{
    if (T < 0 || P <= 0 || V <= 0) return A3PO_E_SIZE;
    if (T == 0) return A3PO_OK;
    if (!partials || !chosen || !logp_out) return A3PO_E_NULL;
    if (!aligned(partials, 16)) return A3PO_E_ALIGN;
    const hipError_t e = launch_shard_combine(partials, P, T, chosen, V, logp_out, lse_out, entropy_out, nullptr,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}

int a3po_shard_loss_bwd(const void *logits_shard, a3po_dtype dt, int64_t T, int64_t Vs, int64_t ld, int64_t v0,
                        int64_t V, const int32_t *chosen, const float *logp_theta, const float *lse,
                        const float *logp_behav, const int32_t *versions, int32_t current_version,
                        const float *advantages, const uint8_t *loss_mask, float clip_eps, float denom,
                        void *dlogits_shard, float *logp_prox_out, float *loss_out, a3po_stats *stats_out,
                        void *workspace, size_t workspace_bytes, void *stream, const a3po_loss_options *opt)
{
    const a3po_loss_options none = {};
    const a3po_loss_options &o = opt ? *opt : none;
    if (int rc = check_logits(logits_shard, (int)dt, T, Vs, ld)) return rc;
    if (v0 < 0 || V <= 0 || v0 + Vs > V || V > (int64_t)0x7FFFFFFF) return A3PO_E_SIZE;
    if (T > kQueueMaxItems || shard_bwd_queue_items((int)dt, T, Vs) > kQueueMaxItems) return A3PO_E_SIZE;
    if (!(clip_eps >= 0.0f && clip_eps < 1.0f) || std::isnan(denom)) return A3PO_E_VALUE;
    if (o.prox_mode < A3PO_PROX_INTERP || o.prox_mode > A3PO_PROX_BEHAV || (o.accumulate != 0 && o.accumulate != 1))
        return A3PO_E_VALUE;
    if (!loss_out) return A3PO_E_NULL;
    if (T > 0 && (!dlogits_shard || !chosen || !logp_theta || !lse || !logp_behav || !advantages || !loss_mask))
        return A3PO_E_NULL;
    if (T > 0 && o.prox_mode == A3PO_PROX_INTERP && !versions) return A3PO_E_NULL;
    if (T > 0 && o.prox_mode == A3PO_PROX_GIVEN && !o.logp_prox_in) return A3PO_E_NULL;
    if (!aligned(dlogits_shard, dt == A3PO_F32 ? 4 : 2)) return A3PO_E_ALIGN;
    const WsLayout lay = loss_ws_layout(T);
    if (!workspace || workspace_bytes < lay.total) return A3PO_E_WORKSPACE;
    if (!aligned(workspace, 256)) return A3PO_E_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    LossArgs a;
    a.z = logits_shard;
    a.dz = dlogits_shard;
    a.dt = (int)dt;
    a.T = T;
    a.V = V;  // the prep kernel validates chosen ids against the full vocabulary
    a.ld = ld;
    a.chosen = chosen;
    a.lb = logp_behav;
    a.versions = versions;
    a.current_version = current_version;
    a.adv = advantages;
    a.mask = loss_mask;
    a.clip_eps = clip_eps;
    a.denom = denom;
    a.logp_out = nullptr;
    a.prox_out = logp_prox_out;
    a.loss_out = loss_out;
    a.stats_out = stats_out;
    a.prox_mode = o.prox_mode;
    a.prox_in = o.logp_prox_in;
    a.iw_out = o.iw_out;
    a.clipped_out = o.clipped_out;
    a.denom_dev = o.denom_dev;
    a.accumulate = o.accumulate;
    carve_loss_ws(a, workspace, T);
    if (launch_loss_prep(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    LossArgs b = a;
    b.V = Vs;  // the row kernel walks the shard's columns
    if (launch_shard_bwd_rows(b, v0, logp_theta, lse, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (launch_loss_finish(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    return A3PO_OK;
}

}  // extern "C"
