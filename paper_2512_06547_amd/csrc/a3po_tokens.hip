// Per-token kernels (O(T) work): mask count before the row kernel, fixed-order loss and
// statistics reduction after it, the stand-alone proximal interpolation, GRPO advantages,
// histograms of per-token quantities.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

constexpr int kTokThreads = 1024;
constexpr int kTokWaves = kTokThreads / kWave;

// Counts of a range of tokens: those that enter the loss (mask != 0 and a valid chosen id), and those with
// mask != 0 and an id outside [0, V).
struct PrepPartial {
    long long cnt, bad;
};

// Packs the inputs of tokens [t_begin, t_end) into one 16-byte record each for the row kernel (y = -1 when the
// token does not enter the loss) and counts them; the totals of the workgroup are returned to thread 0.
__device__ __forceinline__ PrepPartial pack_records(const int32_t *chosen, const uint8_t *mask, const float *lb,
                                                    const int32_t *versions, const float *adv, const float *prox_in,
                                                    int64_t t_begin, int64_t t_end, int64_t V, TokenRecord *records)
{
    __shared__ long long s_cnt[kTokWaves], s_bad[kTokWaves];
    long long cnt = 0, bad = 0;
    for (int64_t t = t_begin + threadIdx.x; t < t_end; t += kTokThreads) {
        const bool m = mask[t] != 0;
        const int32_t y = chosen[t];
        const bool ok = y >= 0 && (int64_t)y < V;
        cnt += (m && ok) ? 1 : 0;
        bad += (m && !ok) ? 1 : 0;
        TokenRecord r;
        r.y = (m && ok) ? y : -1;
        // a given proximal log-prob rides in the version slot; the coupled objective needs neither
        r.ver = prox_in ? __float_as_int(prox_in[t]) : (versions ? versions[t] : 0);
        r.lb = lb[t];
        r.A = adv[t];
        records[t] = r;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        cnt += __shfl_xor(cnt, off, kWave);
        bad += __shfl_xor(bad, off, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) {
        s_cnt[wave] = cnt;
        s_bad[wave] = bad;
    }
    __syncthreads();
    PrepPartial p = {0, 0};
    if (threadIdx.x == 0) {
        for (int w = 0; w < kTokWaves; ++w) {
            p.cnt += s_cnt[w];
            p.bad += s_bad[w];
        }
    }
    return p;
}

// Header of a call: 1/N with N the number of counted tokens, or the caller's denominator when it is positive;
// the counts for the statistics; the row kernel's work queue starts empty.
__device__ __forceinline__ void write_header(PrepPartial total, float denom, WsHeader *hdr)
{
    const float n = denom > 0.0f ? denom : (float)total.cnt;
    hdr->inv_n = n > 0.0f ? 1.0f / n : 0.0f;
    hdr->n_as_float = n;
    hdr->n_counted = total.cnt;
    hdr->n_bad = total.bad;
    *row_queue_of(hdr) = 0u;
}

// One workgroup does both (short batches).
__global__ __launch_bounds__(kTokThreads) void loss_prep_kernel(const int32_t *chosen, const uint8_t *mask,
                                                                const float *lb, const int32_t *versions,
                                                                const float *adv, const float *prox_in, int64_t T,
                                                                int64_t V, float denom, const float *denom_dev,
                                                                WsHeader *hdr, TokenRecord *records)
{
    const PrepPartial total = pack_records(chosen, mask, lb, versions, adv, prox_in, 0, T, V, records);
    if (threadIdx.x == 0) write_header(total, denom_dev ? *denom_dev : denom, hdr);
}

// Long batches: workgroup b packs the records of tokens [b, b+1) * per_block and leaves its counts in the
// scratch area; a one-workgroup kernel adds the counts (integers: any order) and writes the header.
__global__ __launch_bounds__(kTokThreads) void loss_prep_records_kernel(const int32_t *chosen, const uint8_t *mask,
                                                                        const float *lb, const int32_t *versions,
                                                                        const float *adv, const float *prox_in,
                                                                        int64_t T, int64_t V, TokenRecord *records,
                                                                        PrepPartial *partial, int64_t per_block)
{
    const int64_t t_begin = (int64_t)blockIdx.x * per_block;
    const PrepPartial p =
        pack_records(chosen, mask, lb, versions, adv, prox_in, t_begin, min(T, t_begin + per_block), V, records);
    if (threadIdx.x == 0) partial[blockIdx.x] = p;
}

__global__ __launch_bounds__(kTokMaxBlocks) void loss_prep_header_kernel(const PrepPartial *partial, int nblocks,
                                                                        float denom, const float *denom_dev,
                                                                        WsHeader *hdr)
{
    __shared__ long long s_cnt[kTokMaxBlocks / kWave], s_bad[kTokMaxBlocks / kWave];
    long long cnt = 0, bad = 0;
    if ((int)threadIdx.x < nblocks) {
        cnt = partial[threadIdx.x].cnt;
        bad = partial[threadIdx.x].bad;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        cnt += __shfl_xor(cnt, off, kWave);
        bad += __shfl_xor(bad, off, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) {
        s_cnt[wave] = cnt;
        s_bad[wave] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        PrepPartial total = {0, 0};
        for (int w = 0; w < kTokMaxBlocks / kWave; ++w) {
            total.cnt += s_cnt[w];
            total.bad += s_bad[w];
        }
        write_header(total, denom_dev ? *denom_dev : denom, hdr);
    }
}

// Totals of the finish pass over a range of tokens.
struct FinishTotals {
    double sum, esum;     // sum of obj and of the entropies over counted tokens
    long long clip, neg;  // clipped tokens, tokens with negative staleness
    float lo, hi;         // extrema of the importance weight
};

static_assert(sizeof(FinishTotals) <= 64 && sizeof(PrepPartial) <= 64, "a partial is at most 64 bytes of the scratch area");

// loss_out / stats_out from the totals of the whole call (overwritten, or merged into what earlier micro-batches of
// the same update left there)
__device__ __forceinline__ void write_loss_and_stats(const FinishTotals &tot, bool have_entropy, const WsHeader *hdr,
                                                     float *loss_out, a3po_stats *stats, int accumulate)
{
    const float share = (float)(-(tot.sum * (double)hdr->inv_n));
    *loss_out = accumulate ? *loss_out + share : share;
    if (!stats) return;
    a3po_stats o;
    o.n_tokens = hdr->n_counted;
    o.n_clipped = tot.clip;
    o.n_bad_index = hdr->n_bad;
    o.n_negative_staleness = tot.neg;
    o.iw_min = tot.lo;
    o.iw_max = tot.hi;
    o.entropy_mean = (have_entropy && hdr->n_counted > 0) ? (float)(tot.esum / (double)hdr->n_counted) : 0.0f;
    o.reserved = 0.0f;
    if (accumulate) {
        const a3po_stats p = *stats;
        const long long n = p.n_tokens + o.n_tokens;
        o.entropy_mean = (have_entropy && n > 0)
                             ? (float)(((double)p.entropy_mean * (double)p.n_tokens + tot.esum) / (double)n)
                             : 0.0f;
        o.n_tokens = n;
        o.n_clipped += p.n_clipped;
        o.n_bad_index += p.n_bad_index;
        o.n_negative_staleness += p.n_negative_staleness;
        o.iw_min = fminf(o.iw_min, p.iw_min);
        o.iw_max = fmaxf(o.iw_max, p.iw_max);
    }
    *stats = o;
}

// loss = -(1/N) sum over counted tokens of obj, accumulated in double in a fixed order
// (thread-strided partials, then a fixed tree), so repeated runs agree bit for bit.
// ent (nullable): per-token entropies the row kernel wrote; their mean over counted tokens goes to
// the statistics.  iw_out / clipped_out (nullable): per-token copies for the caller.
// partial == nullptr: one workgroup covers all T tokens and writes loss and statistics itself.  Otherwise workgroup b
// covers tokens [b, b+1) * per_block and leaves its totals in partial[b] for loss_finish_final_kernel.
__global__ __launch_bounds__(kTokThreads) void loss_finish_kernel(const float *obj, const float *iw, const uint8_t *flags,
                                                                  const float *ent, int64_t T, const WsHeader *hdr,
                                                                  float *loss_out, a3po_stats *stats, float *iw_out,
                                                                  uint8_t *clipped_out, int accumulate,
                                                                  FinishTotals *partial, int64_t per_block)
{
    const int64_t t_begin = partial ? (int64_t)blockIdx.x * per_block : 0;
    const int64_t t_end = partial ? min(T, t_begin + per_block) : T;
    __shared__ double s_sum[kTokWaves], s_ent[kTokWaves];
    __shared__ long long s_clip[kTokWaves], s_neg[kTokWaves];
    __shared__ float s_min[kTokWaves], s_max[kTokWaves];
    double sum = 0.0, esum = 0.0;
    long long clip = 0, neg = 0;
    float lo = INFINITY, hi = -INFINITY;
    // kFinishUnroll tokens' loads are in flight before the first is used (one workgroup: latency, not bandwidth);
    // the order of a thread's additions is that of its tokens, whatever the unroll
    constexpr int kFinishUnroll = 8;
    for (int64_t t0 = t_begin + threadIdx.x; t0 < t_end; t0 += (int64_t)kFinishUnroll * kTokThreads) {
        uint8_t f[kFinishUnroll];
        float o[kFinishUnroll], w[kFinishUnroll], h[kFinishUnroll];
#pragma unroll
        for (int u = 0; u < kFinishUnroll; ++u) {
            const int64_t t = t0 + (int64_t)u * kTokThreads;
            f[u] = 0;
            o[u] = w[u] = h[u] = 0.0f;
            if (t < t_end) {
                f[u] = flags[t];
                o[u] = obj[t];
                w[u] = iw[t];
                if (ent) h[u] = ent[t];
            }
        }
#pragma unroll
        for (int u = 0; u < kFinishUnroll; ++u) {
            const int64_t t = t0 + (int64_t)u * kTokThreads;
            if (t >= t_end) continue;
            if (iw_out) iw_out[t] = (f[u] & kFlagCounted) ? w[u] : 0.0f;
            if (clipped_out) clipped_out[t] = (f[u] & kFlagClipped) ? 1 : 0;
            if (f[u] & kFlagCounted) {
                sum += (double)o[u];
                if (ent) esum += (double)h[u];
                clip += (f[u] & kFlagClipped) ? 1 : 0;
                neg += (f[u] & kFlagNegStale) ? 1 : 0;
                lo = fminf(lo, w[u]);
                hi = fmaxf(hi, w[u]);
            }
        }
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        sum += __shfl_xor(sum, off, kWave);
        esum += __shfl_xor(esum, off, kWave);
        clip += __shfl_xor(clip, off, kWave);
        neg += __shfl_xor(neg, off, kWave);
        lo = fminf(lo, __shfl_xor(lo, off, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) {
        s_sum[wave] = sum;
        s_ent[wave] = esum;
        s_clip[wave] = clip;
        s_neg[wave] = neg;
        s_min[wave] = lo;
        s_max[wave] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        FinishTotals tot = {0.0, 0.0, 0, 0, INFINITY, -INFINITY};
        for (int w = 0; w < kTokWaves; ++w) {
            tot.sum += s_sum[w];
            tot.esum += s_ent[w];
            tot.clip += s_clip[w];
            tot.neg += s_neg[w];
            tot.lo = fminf(tot.lo, s_min[w]);
            tot.hi = fmaxf(tot.hi, s_max[w]);
        }
        if (partial) partial[blockIdx.x] = tot;
        else write_loss_and_stats(tot, ent != nullptr, hdr, loss_out, stats, accumulate);
    }
}

// Long batches: the kernel above runs on several workgroups (workgroup b over tokens [b, b+1) * per_block,
// totals to the scratch area); this one adds the workgroups' totals in a fixed tree and writes loss and statistics.
__global__ __launch_bounds__(kTokMaxBlocks) void loss_finish_final_kernel(const FinishTotals *partial, int nblocks,
                                                                         int have_entropy, const WsHeader *hdr,
                                                                         float *loss_out, a3po_stats *stats,
                                                                         int accumulate)
{
    __shared__ FinishTotals s_tot[kTokMaxBlocks / kWave];
    FinishTotals t = {0.0, 0.0, 0, 0, INFINITY, -INFINITY};
    if ((int)threadIdx.x < nblocks) t = partial[threadIdx.x];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        t.sum += __shfl_xor(t.sum, off, kWave);
        t.esum += __shfl_xor(t.esum, off, kWave);
        t.clip += __shfl_xor(t.clip, off, kWave);
        t.neg += __shfl_xor(t.neg, off, kWave);
        t.lo = fminf(t.lo, __shfl_xor(t.lo, off, kWave));
        t.hi = fmaxf(t.hi, __shfl_xor(t.hi, off, kWave));
    }
    if ((threadIdx.x & (kWave - 1)) == 0) s_tot[threadIdx.x / kWave] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        FinishTotals tot = {0.0, 0.0, 0, 0, INFINITY, -INFINITY};
        for (int w = 0; w < kTokMaxBlocks / kWave; ++w) {
            tot.sum += s_tot[w].sum;
            tot.esum += s_tot[w].esum;
            tot.clip += s_tot[w].clip;
            tot.neg += s_tot[w].neg;
            tot.lo = fminf(tot.lo, s_tot[w].lo);
            tot.hi = fmaxf(tot.hi, s_tot[w].hi);
        }
        write_loss_and_stats(tot, have_entropy != 0, hdr, loss_out, stats, accumulate);
    }
}

// Counted tokens (mask != 0 and a valid chosen id) of a mini-batch, as the denominator of its micro-batches.
__global__ __launch_bounds__(kTokThreads) void count_tokens_kernel(const int32_t *chosen, const uint8_t *mask, int64_t T,
                                                                   int64_t V, float *denom_out, int64_t *count_out)
{
    __shared__ long long s_cnt[kTokWaves];
    long long cnt = 0;
    for (int64_t t = threadIdx.x; t < T; t += kTokThreads) {
        const int32_t y = chosen[t];
        cnt += (mask[t] != 0 && y >= 0 && (int64_t)y < V) ? 1 : 0;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) s_cnt[threadIdx.x / kWave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long c = 0;
        for (int w = 0; w < kTokWaves; ++w) c += s_cnt[w];
        *denom_out = (float)c;
        if (count_out) *count_out = c;
    }
}

// Histogram over explicit edges: slot k of a value = number of edges <= it (0: below the first edge,
// nbins + 1: at or above the last), slot nbins + 2 for NaN.  Edges and per-workgroup counts live in LDS;
// integer atomics only, so the result does not depend on the order of arrival.
constexpr int kHistThreads = 256;
constexpr int kHistMaxBlocks = 512;

__global__ void histogram_clear_kernel(int64_t *counts, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counts[i] = 0;
}

__global__ __launch_bounds__(kHistThreads) void histogram_kernel(const float *__restrict__ values,
                                                                 const uint8_t *__restrict__ select, int64_t T,
                                                                 const float *__restrict__ edges, int nbins,
                                                                 unsigned long long *__restrict__ counts)
{
    __shared__ float s_edge[A3PO_HIST_MAX_BINS + 1];
    __shared__ unsigned long long s_cnt[A3PO_HIST_MAX_BINS + 3];
    for (int i = threadIdx.x; i <= nbins; i += kHistThreads) s_edge[i] = edges[i];
    for (int i = threadIdx.x; i < nbins + 3; i += kHistThreads) s_cnt[i] = 0ull;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    for (int64_t t = (int64_t)blockIdx.x * kHistThreads + threadIdx.x; t < T; t += stride) {
        if (select && select[t] == 0) continue;
        const float v = values[t];
        int lo = 0, hi = nbins + 1;  // lo ends as the number of edges <= v
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_edge[mid] <= v) lo = mid + 1;
            else hi = mid;
        }
        atomicAdd(&s_cnt[v != v ? nbins + 2 : lo], 1ull);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbins + 3; i += kHistThreads)
        if (s_cnt[i]) atomicAdd(&counts[i], s_cnt[i]);
}

hipError_t launch_histogram(const float *values, const uint8_t *select, int64_t T, const float *edges, int nbins,
                            bool accumulate, int64_t *counts, hipStream_t s)
{
    if (!accumulate) {
        hipLaunchKernelGGL(histogram_clear_kernel, dim3((nbins + 3 + 255) / 256), dim3(256), 0, s, counts, nbins + 3);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (T == 0) return hipSuccess;
    const int64_t want = (T + kHistThreads * 8 - 1) / (kHistThreads * 8);
    const unsigned grid = (unsigned)(want < kHistMaxBlocks ? want : kHistMaxBlocks);
    hipLaunchKernelGGL(histogram_kernel, dim3(grid), dim3(kHistThreads), 0, s, values, select, T, edges, nbins,
                       reinterpret_cast<unsigned long long *>(counts));
    return hipGetLastError();
}

// Eq. 3 with the coefficient of Eq. 4, element-wise.
__global__ void proximal_interp_kernel(const float *lb, const float *lt, const int32_t *versions,
                                       int32_t current_version, int64_t T, float *lp, float *alpha_out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int64_t d = (int64_t)current_version - (int64_t)versions[t];
    const float alpha = d >= 1 ? 1.0f / (float)d : 1.0f;
    lp[t] = alpha * lb[t] + (1.0f - alpha) * lt[t];
    if (alpha_out) alpha_out[t] = alpha;
}

// GRPO group-normalised advantage of the sequence each token belongs to.
__global__ void grpo_advantages_kernel(const float *rewards, int64_t S, int32_t G, float eps_adv, const int32_t *seq_id,
                                       int64_t T, float *adv)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int32_t s = seq_id[t];
    if (s < 0 || (int64_t)s >= S) {
        adv[t] = 0.0f;
        return;
    }
    const int64_t g0 = ((int64_t)s / G) * G;
    double mu = 0.0;
    for (int32_t k = 0; k < G; ++k) mu += (double)rewards[g0 + k];
    mu /= (double)G;
    double var = 0.0;
    for (int32_t k = 0; k < G; ++k) {
        const double c = (double)rewards[g0 + k] - mu;
        var += c * c;
    }
    var /= (double)G;
    adv[t] = (float)(((double)rewards[s] - mu) / (sqrt(var) + (double)eps_adv));
}

// Workgroups of the O(T) kernels and the tokens each takes: one workgroup up to kTokSingleMax tokens (a second
// launch for the partials costs more than it saves there: one workgroup takes about 4 us + 0.4 us per 1,000
// tokens, the split pair about 11 us), else one per kTokBlockTokens up to the kTokMaxBlocks partials the scratch
// area holds, beyond that equal shares of the batch.
constexpr int64_t kTokSingleMax = 16384;
struct TokSplit {
    int blocks;
    int64_t per_block;
};
static TokSplit tok_split(int64_t T)
{
    const int64_t want = T <= kTokSingleMax ? 1 : (T + kTokBlockTokens - 1) / kTokBlockTokens;
    TokSplit sp;
    sp.blocks = (int)(want > kTokMaxBlocks ? kTokMaxBlocks : want);
    sp.per_block = T > 0 ? (T + sp.blocks - 1) / sp.blocks : 1;
    return sp;
}

hipError_t launch_loss_prep(const LossArgs &a, hipStream_t s)
{
    const int32_t *ver = a.prox_mode == A3PO_PROX_INTERP ? a.versions : nullptr;
    const float *prox = a.prox_mode == A3PO_PROX_GIVEN ? a.prox_in : nullptr;
    const TokSplit sp = tok_split(a.T);
    const int nb = sp.blocks;
    if (nb == 1) {
        hipLaunchKernelGGL(loss_prep_kernel, dim3(1), dim3(kTokThreads), 0, s, a.chosen, a.mask, a.lb, ver, a.adv, prox,
                           a.T, a.V, a.denom, a.denom_dev, reinterpret_cast<WsHeader *>(a.ws_header), a.ws_records);
        return hipGetLastError();
    }
    PrepPartial *part = reinterpret_cast<PrepPartial *>(a.ws_scratch);
    hipLaunchKernelGGL(loss_prep_records_kernel, dim3(nb), dim3(kTokThreads), 0, s, a.chosen, a.mask, a.lb, ver, a.adv,
                       prox, a.T, a.V, a.ws_records, part, sp.per_block);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(loss_prep_header_kernel, dim3(1), dim3(kTokMaxBlocks), 0, s, part, nb, a.denom, a.denom_dev,
                       reinterpret_cast<WsHeader *>(a.ws_header));
    return hipGetLastError();
}

hipError_t launch_count_tokens(const int32_t *chosen, const uint8_t *mask, int64_t T, int64_t V, float *denom_out,
                               int64_t *count_out, hipStream_t s)
{
    hipLaunchKernelGGL(count_tokens_kernel, dim3(1), dim3(kTokThreads), 0, s, chosen, mask, T, V, denom_out, count_out);
    return hipGetLastError();
}

__global__ void reset_row_queue_kernel(void *ws_header) { *row_queue_of(ws_header) = 0u; }

hipError_t launch_reset_row_queue(void *ws_header, hipStream_t s)
{
    hipLaunchKernelGGL(reset_row_queue_kernel, dim3(1), dim3(1), 0, s, ws_header);
    return hipGetLastError();
}

hipError_t launch_loss_finish(const LossArgs &a, hipStream_t s)
{
    const WsHeader *hdr = reinterpret_cast<const WsHeader *>(a.ws_header);
    const TokSplit sp = tok_split(a.T);
    const int nb = sp.blocks;
    FinishTotals *part = nb == 1 ? nullptr : reinterpret_cast<FinishTotals *>(a.ws_scratch);
    hipLaunchKernelGGL(loss_finish_kernel, dim3(nb), dim3(kTokThreads), 0, s, a.ws_obj, a.ws_iw, a.ws_flags, a.ent_out,
                       a.T, hdr, a.loss_out, a.stats_out, a.iw_out, a.clipped_out, a.accumulate, part, sp.per_block);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nb == 1) return e;
    hipLaunchKernelGGL(loss_finish_final_kernel, dim3(1), dim3(kTokMaxBlocks), 0, s, part, nb, a.ent_out != nullptr, hdr,
                       a.loss_out, a.stats_out, a.accumulate);
    return hipGetLastError();
}

hipError_t launch_proximal_interp(const float *lb, const float *lt, const int32_t *versions, int32_t current_version,
                                  int64_t T, float *lp, float *alpha, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const unsigned grid = (unsigned)((T + 255) / 256);
    hipLaunchKernelGGL(proximal_interp_kernel, dim3(grid), dim3(256), 0, s, lb, lt, versions, current_version, T, lp,
                       alpha);
    return hipGetLastError();
}

hipError_t launch_grpo_advantages(const float *rewards, int64_t S, int32_t G, float eps_adv, const int32_t *seq_id,
                                  int64_t T, float *adv, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const unsigned grid = (unsigned)((T + 255) / 256);
    hipLaunchKernelGGL(grpo_advantages_kernel, dim3(grid), dim3(256), 0, s, rewards, S, G, eps_adv, seq_id, T, adv);
    return hipGetLastError();
}

}  // namespace a3po
