// Token log-probs straight from hidden states and the LM-head weight: z = h W^T is produced tile by tile on the
// matrix cores (a3po_gemm.hip, with the vocabulary on the row side and the tokens on the column side of the
// tile) and folded into a running (max, sum) per token as each tile leaves the accumulators, so the [T, V]
// logits never exist in memory.  A small kernel then merges the partials of the workgroups that shared a
// token, adds the chosen logit (a separate dot product) and writes log pi.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

// z[t, y_t] = h[t, :] . W[y_t, :] in fp32, one wavefront per token; then
// lse_t from the partials of the workgroups that swept this token and log pi = z_y - lse.
__global__ __launch_bounds__(256) void lmhead_finish_kernel(const uint16_t *__restrict__ W,
                                                            const uint16_t *__restrict__ h, int64_t T, int64_t H,
                                                            int64_t V, const int32_t *__restrict__ chosen,
                                                            const float2 *__restrict__ partial, int64_t partial_stride,
                                                            int nparts, float *logp, float *lse_out, DynCount count)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= dyn_extent(count, T)) return;
    const int32_t y = chosen[t];
    const bool ok = y >= 0 && (int64_t)y < V;
    float dot = 0.0f;
    if (ok) {
        const uint16_t *hr = h + t * H, *wr = W + (int64_t)y * H;
        for (int64_t k = (int64_t)lane * 8; k + 8 <= H; k += 64 * 8) {
            float a[8], b[8];
            unpack<Bf16>(*reinterpret_cast<const uint4 *>(hr + k), a);
            unpack<Bf16>(*reinterpret_cast<const uint4 *>(wr + k), b);
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(a[e], b[e], dot);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, kWave);
    }
    if (lane == 0) {
        MaxSum tot = {kNegFloor, 0.0f};
        for (int p = 0; p < nparts; ++p) {
            const float2 q = partial[(int64_t)p * partial_stride + t];
            tot = combine(tot, MaxSum{q.x, q.y});
        }
        const float log_s = logf(tot.s);
        if (lse_out) lse_out[t] = tot.m + log_s;
        logp[t] = ok ? (dot - tot.m) - log_s : 0.0f;
    }
}

size_t lmhead_workspace_bytes(int64_t T)
{
    const size_t t = (size_t)(T > 0 ? T : 0);
    return ((t * kGemmMaxPartialSlots * sizeof(float2) + 255) / 256) * 256 + 256;
}

hipError_t launch_lmhead_lse_finish(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                    const int32_t *chosen, const float2 *partial, int64_t partial_stride, float *logp,
                                    float *lse, hipStream_t s, DynCount count)
{
    const unsigned grid = (unsigned)((T + 3) / 4);
    hipLaunchKernelGGL(lmhead_finish_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<const uint16_t *>(weight),
                       reinterpret_cast<const uint16_t *>(hidden), T, H, V, chosen, partial, partial_stride,
                       (int)gemm_partial_slots(), logp, lse, count);
    return hipGetLastError();
}

hipError_t launch_fused_lmhead_logprob(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                       const int32_t *chosen, float *logp, float *lse, void *workspace, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    GemmArgs g = {};
    g.A = reinterpret_cast<const uint16_t *>(weight);
    g.lda = H;
    g.B = reinterpret_cast<const uint16_t *>(hidden);
    g.ldb = H;
    g.M = V;
    g.N = T;
    g.K = H;
    g.partial = reinterpret_cast<float2 *>(workspace);
    g.partial_stride = T;
    hipError_t e = launch_gemm_nt(g, kEpiLse, s);
    if (e != hipSuccess) return e;
    return launch_lmhead_lse_finish(hidden, weight, T, H, V, chosen, g.partial, T, logp, lse, s);
}

}  // namespace a3po
