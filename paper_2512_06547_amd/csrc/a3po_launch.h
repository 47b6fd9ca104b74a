// Host-side launch interface between the C ABI (a3po_api.hip) and the kernel files.
#pragma once

#include <mutex>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "a3po.h"

namespace a3po {

struct TokenRecord;

struct LossArgs {
    const void *z;
    void *dz;
    int dt;  // a3po_dtype
    int64_t T, V, ld;
    const int32_t *chosen;
    const float *lb;
    const int32_t *versions;
    int32_t current_version;
    const float *adv;
    const uint8_t *mask;
    float clip_eps;
    float denom;
    float *logp_out;
    float *prox_out;  // nullable
    float *loss_out;
    a3po_stats *stats_out;  // nullable
    int prox_mode = 0;               // a3po_prox_mode
    const float *prox_in = nullptr;  // [T], A3PO_PROX_GIVEN only
    float *ent_out = nullptr;        // [T] policy entropy, nullable
    float *iw_out = nullptr;         // [T] importance weights, nullable
    uint8_t *clipped_out = nullptr;  // [T] clip decisions, nullable
    const float *denom_dev = nullptr;  // device [1], overrides denom when set
    int accumulate = 0;              // add to loss_out / stats_out instead of overwriting
    // workspace carve-up
    void *ws_header;
    TokenRecord *ws_records;  // [T], written by the prep kernel
    float *ws_obj;
    float *ws_iw;
    uint8_t *ws_flags;
    void *ws_scratch;               // kLossScratchBytes: per-workgroup partials of the prep and finish kernels
};

// Workspace of the loss path: header | TokenRecord[T] (16 bytes each) | obj[T] | iw[T] | flags[T] | scratch
struct LossWsLayout {
    size_t records, obj, iw, flags, scratch, total;
};

// The O(T) kernels before and after the row kernel run on up to kTokMaxBlocks workgroups of kTokBlockTokens tokens
// each (one workgroup for short batches); each leaves a partial of at most 64 bytes in the scratch area.
constexpr int kTokMaxBlocks = 256;
constexpr int kTokBlockTokens = 2048;
constexpr size_t kLossScratchBytes = (size_t)kTokMaxBlocks * 64;
inline LossWsLayout loss_ws_layout(int64_t T)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const size_t t = (size_t)(T > 0 ? T : 0);
    LossWsLayout l;
    l.records = 256;
    l.obj = l.records + up(t * 16);
    l.iw = l.obj + up(t * sizeof(float));
    l.flags = l.iw + up(t * sizeof(float));
    l.scratch = l.flags + up(t);
    l.total = l.scratch + kLossScratchBytes;
    return l;
}

// points the workspace fields of `a` into a workspace laid out for T tokens
inline void carve_loss_ws(LossArgs &a, void *workspace, int64_t T)
{
    char *ws = static_cast<char *>(workspace);
    const LossWsLayout lay = loss_ws_layout(T);
    a.ws_header = ws;
    a.ws_records = reinterpret_cast<TokenRecord *>(ws + lay.records);
    a.ws_obj = reinterpret_cast<float *>(ws + lay.obj);
    a.ws_iw = reinterpret_cast<float *>(ws + lay.iw);
    a.ws_flags = reinterpret_cast<uint8_t *>(ws + lay.flags);
    a.ws_scratch = ws + lay.scratch;
}

// true when the single-pass register-resident kernel can take these rows
bool rows_fit_on_chip(int dt, int64_t V, int64_t ld, const void *z, const void *dz);

hipError_t launch_loss_prep(const LossArgs &a, hipStream_t s);
hipError_t launch_loss_rows(const LossArgs &a, hipStream_t s);
hipError_t launch_loss_finish(const LossArgs &a, hipStream_t s);
hipError_t launch_count_tokens(const int32_t *chosen, const uint8_t *mask, int64_t T, int64_t V, float *denom_out,
                               int64_t *count_out, hipStream_t s);
hipError_t launch_histogram(const float *values, const uint8_t *select, int64_t T, const float *edges, int nbins,
                            bool accumulate, int64_t *counts, hipStream_t s);
hipError_t launch_reset_row_queue(void *ws_header, hipStream_t s);  // before re-running the row kernel on one header

hipError_t launch_token_logprobs(const void *z, int dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                                 float *logp, float *lse, void *chosen_logit, float *ent, hipStream_t s);
hipError_t launch_proximal_interp(const float *lb, const float *lt, const int32_t *versions, int32_t current_version,
                                  int64_t T, float *lp, float *alpha, hipStream_t s);
hipError_t launch_grpo_advantages(const float *rewards, int64_t S, int32_t G, float eps_adv, const int32_t *seq_id,
                                  int64_t T, float *adv, hipStream_t s);

// records (nullable): rows whose record says "not counted" are skipped (partials) / get zeros (combine)
hipError_t launch_shard_partials(const void *z, int dt, int64_t T, int64_t Vs, int64_t ld, const int32_t *chosen,
                                 int64_t v0, a3po_shard_partial *out, const TokenRecord *records, hipStream_t s);
hipError_t launch_shard_combine(const a3po_shard_partial *parts, int32_t P, int64_t T, const int32_t *chosen, int64_t V,
                                float *logp, float *lse, float *ent, const TokenRecord *records, hipStream_t s);
// the loss rows in three streaming passes (partials, merge, gradient bursts) for rows that do not fit on chip
// The row kernel and the gradient bursts hand out work through a 32-bit counter: item index = grid size + number
// of claims so far, and every workgroup makes one claim past the end.  Item counts above this bound are refused
// by the entry points (rows for the register-resident kernel, bursts for the streaming one).
constexpr int64_t kQueueMaxItems = ((int64_t)1 << 32) - ((int64_t)1 << 16);
int64_t shard_bwd_queue_items(int dt, int64_t T, int64_t Vs);  // bursts launch_shard_bwd_rows would queue (0: no queue)
// a.V is the shard width here; a.ws_records must come from a prep launch made with the full vocabulary size
hipError_t launch_shard_bwd_rows(const LossArgs &a, int64_t v0, const float *logp_theta, const float *lse, hipStream_t s);

// ---- bfloat16 contraction on the matrix cores (a3po_gemm.hip): C[M, N] = A[M, K] B[N, K]^T ------------------
enum GemmEpilogue {
    kEpiLse = 0,        // running (max, sum) per column n over the rows m -> partial; C untouched
    kEpiLseStore = 1,   // the same, and C (float) = the product
    kEpiStoreBf16 = 2,  // C (bfloat16) = the product
    kEpiAccumF32 = 3    // C (float) = the product, or += when accumulate is set
};

// An extent that is only known on the device when the launch is queued (the number of tokens that enter the loss):
// extent = clamp(*n - offset, 0, cap), or the host's value when n is null.
struct DynCount {
    const int64_t *n = nullptr;
    int64_t offset = 0, cap = 0;
};
__host__ __device__ inline int64_t dyn_extent(const DynCount &d, int64_t host_value)
{
    if (!d.n) return host_value;
    const int64_t v = *d.n - d.offset;
    return v < 0 ? 0 : (v > d.cap ? d.cap : v);
}

enum GemmDynDim { kDynNone = 0, kDynM = 1, kDynN = 2, kDynK = 3 };

struct GemmArgs {
    const uint16_t *A;  // [M, K] bfloat16, row-major, row stride lda elements (a multiple of 8; 16-byte aligned base)
    int64_t lda;
    const uint16_t *B;  // [N, K] likewise
    int64_t ldb;
    int64_t M, N, K;    // K a multiple of 64 (operands that need it are zero-padded by the caller)
    void *C;            // [M, N] row-major, row stride ldc elements
    int64_t ldc;
    float2 *partial;    // kEpiLse*: [gemm_partial_slots()][partial_stride] (max, sum) per column, merged by the caller
    int64_t partial_stride;
    int a_panel, b_panel;  // the operand is stored in panels instead of rows (see panel_offset): lda / ldb is then the
                           // K extent of the buffer (a multiple of 64), rows are padded to a multiple of 256
    int accumulate;     // kEpiAccumF32
    int transposed;     // kEpiLseStore / kEpiAccumF32: element (m, n) goes to C[n * ldc + m] (C^T row-major, row stride
                        // ldc): a lane's four accumulator values are then 16 contiguous bytes.  Needs M % 4 == 0.
    int dyn_dim;        // GemmDynDim: which of M, N, K is replaced by dyn_extent(dyn, .) on the device (K: rounded up
    DynCount dyn;       // to 128; the host's M, N, K are then upper bounds).  A zero extent makes the launch a no-op.
    int nxcd, ml_count; // filled in by the launcher from the device
};

// Panel layout of a bfloat16 operand of the contraction kernel: the matrix is cut into blocks of 256 rows x 32
// contracted elements - what one stage of the kernel consumes -, each stored as 256 rows x 64 bytes = 16 KiB
// contiguous; blocks of one 256-row band follow each other along K.  A direct load of the kernel (16 rows x 64
// bytes) is then 1 KiB of contiguous memory, eight whole 128-byte lines, instead of 16 half lines a row apart, and
// no power-of-two row stride maps a stage onto a few memory channels.  Element offset of (row, k), kext = K extent:
__host__ __device__ inline int64_t panel_offset(int64_t row, int64_t k, int64_t kext)
{
    return ((row >> 8) * (kext >> 5) + (k >> 5)) * 8192 + (row & 255) * 32 + (k & 31);
}
inline size_t panel_elements(int64_t rows, int64_t kext) { return (size_t)((rows + 255) / 256 * 256) * (size_t)kext; }

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the kernel),
// race-free: the first call on a device sets it under the lock, later calls only look at the flag.  One state
// object per kernel variant.
struct LdsLimitState {
    std::mutex lock;
    bool done[64] = {};
};
inline hipError_t ensure_lds_limit(const void *kernel, int bytes, LdsLimitState &st)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(st.lock);
    if (!st.done[dev]) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        st.done[dev] = true;
    }
    return hipSuccess;
}

struct GemmGrid {
    int nxcd, ml_count, blocks;
};
GemmGrid gemm_grid();
constexpr int kGemmMaxPartialSlots = 64;  // workspaces are sized for this many; gemm_partial_slots() never exceeds it
size_t gemm_partial_slots();
hipError_t launch_gemm_nt(const GemmArgs &g, int epilogue, hipStream_t s);

size_t lmhead_workspace_bytes(int64_t T);
hipError_t launch_fused_lmhead_logprob(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                       const int32_t *chosen, float *logp, float *lse, void *workspace, hipStream_t s);

// merges the (max, sum) partials of a token, adds the chosen logit (a dot product) and writes lse and log pi
// (T is an upper bound when `count` names a device-side token count)
hipError_t launch_lmhead_lse_finish(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                    const int32_t *chosen, const float2 *partial, int64_t partial_stride, float *logp,
                                    float *lse, hipStream_t s, DynCount count = DynCount());

size_t lmhead_bwd_workspace_bytes(int64_t T, int64_t V, int64_t H);

}  // namespace a3po
