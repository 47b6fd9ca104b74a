// Vocabulary-sharded variant of the token log-prob and of the gradient to the logits: the columns of
// the logits are split over P shards (a tensor-parallel LM head), each shard reduces its columns to
// one 16-byte partial per token, the partials of all shards are merged into lse / log pi / entropy,
// and each shard then writes its own slice of the gradient from the merged values.  Between the two
// vocabulary-wide kernels sits whatever exchanges the partials (nothing, on one GPU).
//
// Both kernels stream: a shard row is read once per kernel with 16-byte non-temporal accesses,
// several vectors in flight per thread; nothing is kept between the two kernels except the merged
// per-token scalars, so a shard row crosses HBM three times (read, read, write).
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

// launch shape of the streaming kernels (overridable at build time for tuning sweeps)
#ifndef A3PO_SHARD_THREADS
#define A3PO_SHARD_THREADS 256
#endif
#ifndef A3PO_SHARD_UNROLL
#define A3PO_SHARD_UNROLL 8
#endif
#ifndef A3PO_SHARD_BLOCKS_PER_CU
#define A3PO_SHARD_BLOCKS_PER_CU 8
#endif
constexpr int kShardThreads = A3PO_SHARD_THREADS;
constexpr int kShardWaves = kShardThreads / kWave;
constexpr int kShardUnroll = A3PO_SHARD_UNROLL;  // 16-byte vectors in flight per thread

// ---------------------------------------------------------------------------------------
// partial (max, sum exp, chosen logit if owned, sum exp * z) of one shard, one workgroup per row
template <typename DT>
__global__ __launch_bounds__(kShardThreads) void shard_partials_kernel(const void *z, int64_t T, int64_t Vs, int64_t ld,
                                                                      const int32_t *__restrict__ chosen, int64_t v0,
                                                                      a3po_shard_partial *__restrict__ out, int vec)
{
    constexpr int EPV = DT::kPerVec;
    __shared__ float red[3 * kShardWaves];
    const int tid = threadIdx.x;
    const int nfull = (int)(Vs / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;

    for (int64_t row = blockIdx.x; row < T; row += gridDim.x) {
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        MaxSumU acc;
        seed(acc);
        if (vec) {
            int idx = tid;
            for (; idx + (kShardUnroll - 1) * kShardThreads < nfull; idx += kShardUnroll * kShardThreads) {
                uint4 v[kShardUnroll];
#pragma unroll
                for (int u = 0; u < kShardUnroll; ++u) v[u] = stream_load(in_row + (size_t)(idx + u * kShardThreads) * 16);
#pragma unroll
                for (int u = 0; u < kShardUnroll; ++u) {
                    float f[EPV];
                    unpack<DT>(v[u], f);
                    fold<EPV>(acc, f);
                }
            }
            for (; idx < nfull; idx += kShardThreads) {
                float f[EPV];
                unpack<DT>(stream_load(in_row + (size_t)idx * 16), f);
                fold<EPV>(acc, f);
            }
            for (int64_t j = (int64_t)nfull * EPV + tid; j < Vs; j += kShardThreads) {
                float f[1] = {load_elem<DT>(in_row, j)};
                fold<1>(acc, f);
            }
        } else {
            for (int64_t j = tid; j < Vs; j += kShardThreads) {
                float f[1] = {load_elem<DT>(in_row, j)};
                fold<1>(acc, f);
            }
        }
        const MaxSumU tot = block_allreduce<kShardWaves>(acc, red);
        if (tid == 0) {
            const int64_t yl = (int64_t)chosen[row] - v0;
            a3po_shard_partial p;
            p.max = tot.m;
            p.sum_exp = tot.s;
            p.chosen_logit = (yl >= 0 && yl < Vs) ? load_elem<DT>(in_row, yl) : 0.0f;
            p.sum_exp_z = tot.u;
            out[row] = p;
        }
    }
}

// merge of the P partials of each token (ascending shard order, so the result does not depend on
// the launch shape)
__global__ void shard_combine_kernel(const a3po_shard_partial *__restrict__ parts, int32_t P, int64_t T,
                                     const int32_t *__restrict__ chosen, int64_t V, float *logp, float *lse_out,
                                     float *ent_out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    MaxSumU tot;
    seed(tot);
    float zy = 0.0f;
    for (int32_t p = 0; p < P; ++p) {
        const a3po_shard_partial q = parts[(int64_t)p * T + t];
        tot = combine(tot, MaxSumU{q.max, q.sum_exp, q.sum_exp_z});
        zy += q.chosen_logit;  // exactly one shard owns the chosen column; the others hold 0
    }
    const float lse = tot.m + logf(tot.s);
    const int32_t y = chosen[t];
    const bool ok = y >= 0 && (int64_t)y < V;
    logp[t] = ok ? zy - lse : 0.0f;
    if (lse_out) lse_out[t] = lse;
    if (ent_out) ent_out[t] = entropy_of(tot, lse);
}

// ---------------------------------------------------------------------------------------
// gradient slice of one shard from the merged per-token values:
//   dz[t, j] = g_t ([v0 + j == y_t] - exp(z[t, j] - lse_t)),  g_t from Eq. 2 - Eq. 4 as in the fused kernel.
// Every shard evaluates the per-token terms itself (O(T) work, identical inputs, identical bits).
template <typename DT>
__global__ __launch_bounds__(kShardThreads) void shard_bwd_rows_kernel(
    const void *z, void *dz, int64_t T, int64_t Vs, int64_t ld, int64_t v0, const TokenRecord *__restrict__ records,
    const float *__restrict__ logp_theta, const float *__restrict__ lse_in, int32_t current_version, float clip_eps,
    int prox_mode, const WsHeader *__restrict__ hdr, RowOutputs out, int vec)
{
    constexpr int EPV = DT::kPerVec;
    const int tid = threadIdx.x;
    const int nfull = (int)(Vs / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;
    const float inv_n = hdr->inv_n;

    for (int64_t row = blockIdx.x; row < T; row += gridDim.x) {
        const TokenRecord cur = records[row];
        const int32_t y = cur.y;
        const bool live = y >= 0;
        char *out_row = reinterpret_cast<char *>(dz) + (size_t)row * row_bytes;
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        float g = 0.0f, lse = 0.0f, lt = 0.0f;
        if (live) {
            lse = lse_in[row];
            lt = logp_theta[row];
            const TokenTerms tt =
                token_terms(lt, cur.lb, cur.ver, current_version, cur.A, clip_eps, inv_n, prox_mode);
            g = tt.g;
            if (tid == 0) {
                if (out.prox) out.prox[row] = tt.lp;
                out.obj[row] = tt.obj;
                out.iw[row] = tt.iw;
                out.flags[row] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) |
                                           (tt.negative_staleness ? kFlagNegStale : 0));
            }
        } else if (tid == 0) {
            if (out.prox) out.prox[row] = 0.0f;
            out.obj[row] = 0.0f;
            out.iw[row] = 0.0f;
            out.flags[row] = 0;
        }
        const float neg_g = -g;
        const float nlse = -lse * kLog2e;
        const bool dead = g == 0.0f;  // uniform: zero-fill without reading the row
        if (vec) {
            int idx = tid;
            for (; idx + (kShardUnroll - 1) * kShardThreads < nfull; idx += kShardUnroll * kShardThreads) {
                uint4 v[kShardUnroll];
                if (!dead) {
#pragma unroll
                    for (int u = 0; u < kShardUnroll; ++u)
                        v[u] = stream_load(in_row + (size_t)(idx + u * kShardThreads) * 16);
                }
#pragma unroll
                for (int u = 0; u < kShardUnroll; ++u) {
                    uint4 o = make_uint4(0u, 0u, 0u, 0u);
                    if (!dead) {
                        float f[EPV];
                        unpack<DT>(v[u], f);
#pragma unroll
                        for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw(fmaf(f[e], kLog2e, nlse));
                        o = pack<DT>(f);
                    }
                    stream_store(out_row + (size_t)(idx + u * kShardThreads) * 16, o);
                }
            }
            for (; idx < nfull; idx += kShardThreads) {
                uint4 o = make_uint4(0u, 0u, 0u, 0u);
                if (!dead) {
                    float f[EPV];
                    unpack<DT>(stream_load(in_row + (size_t)idx * 16), f);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw(fmaf(f[e], kLog2e, nlse));
                    o = pack<DT>(f);
                }
                stream_store(out_row + (size_t)idx * 16, o);
            }
            for (int64_t j = (int64_t)nfull * EPV + tid; j < Vs; j += kShardThreads)
                store_elem<DT>(out_row, j, dead ? 0.0f : neg_g * exp2_hw(fmaf(load_elem<DT>(in_row, j), kLog2e, nlse)));
        } else {
            for (int64_t j = tid; j < Vs; j += kShardThreads)
                store_elem<DT>(out_row, j, dead ? 0.0f : neg_g * exp2_hw(fmaf(load_elem<DT>(in_row, j), kLog2e, nlse)));
        }
        // The chosen column, if this shard owns it, gets +g: rewritten by the thread that stored it
        // (same thread, same address: program order).  Its softmax entry is pi_theta(y) = exp(log pi)
        // itself, so the row (possibly already overwritten in place) is not read again.
        const int64_t yl = (int64_t)y - v0;
        if (!dead && yl >= 0 && yl < Vs) {
            int owner;
            if (vec && yl < (int64_t)nfull * EPV) owner = (int)((yl / EPV) % kShardThreads);
            else if (vec) owner = (int)((yl - (int64_t)nfull * EPV) % kShardThreads);
            else owner = (int)(yl % kShardThreads);
            if (tid == owner)
                store_elem<DT>(out_row, yl, neg_g * exp2_hw(lt * kLog2e) + g);
        }
    }
}

// ---------------------------------------------------------------------------------------
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static unsigned shard_grid(int64_t T)
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    const int64_t want = (int64_t)n * A3PO_SHARD_BLOCKS_PER_CU;
    return (unsigned)(T < want ? T : want);
}

hipError_t launch_shard_partials(const void *z, int dt, int64_t T, int64_t Vs, int64_t ld, const int32_t *chosen,
                                 int64_t v0, a3po_shard_partial *out, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(z) && (ld * esz) % 16 == 0;
    if (dt == A3PO_F32)
        hipLaunchKernelGGL((shard_partials_kernel<F32>), dim3(shard_grid(T)), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                           chosen, v0, out, vec);
    else
        hipLaunchKernelGGL((shard_partials_kernel<Bf16>), dim3(shard_grid(T)), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                           chosen, v0, out, vec);
    return hipGetLastError();
}

hipError_t launch_shard_combine(const a3po_shard_partial *parts, int32_t P, int64_t T, const int32_t *chosen, int64_t V,
                                float *logp, float *lse, float *ent, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    hipLaunchKernelGGL(shard_combine_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, parts, P, T, chosen, V,
                       logp, lse, ent);
    return hipGetLastError();
}

hipError_t launch_shard_bwd_rows(const LossArgs &a, int64_t v0, const float *logp_theta, const float *lse, hipStream_t s)
{
    if (a.T == 0) return hipSuccess;
    const int64_t esz = a.dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(a.z) && aligned16(a.dz) && (a.ld * esz) % 16 == 0;
    const RowOutputs out = {nullptr, a.prox_out, a.ws_obj, a.ws_iw, nullptr, a.ws_flags};
    const WsHeader *hdr = reinterpret_cast<const WsHeader *>(a.ws_header);
    if (a.dt == A3PO_F32)
        hipLaunchKernelGGL((shard_bwd_rows_kernel<F32>), dim3(shard_grid(a.T)), dim3(kShardThreads), 0, s, a.z, a.dz,
                           a.T, a.V, a.ld, v0, a.ws_records, logp_theta, lse, a.current_version, a.clip_eps,
                           a.prox_mode, hdr, out, vec);
    else
        hipLaunchKernelGGL((shard_bwd_rows_kernel<Bf16>), dim3(shard_grid(a.T)), dim3(kShardThreads), 0, s, a.z, a.dz,
                           a.T, a.V, a.ld, v0, a.ws_records, logp_theta, lse, a.current_version, a.clip_eps,
                           a.prox_mode, hdr, out, vec);
    return hipGetLastError();
}

}  // namespace a3po
