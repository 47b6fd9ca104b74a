// LM-head projection fused into the token log-prob: z = h W^T is produced tile by tile on the
// matrix cores (v_mfma_f32_32x32x16_bf16) and folded straight into a running (max, sum) per
// token, so the [T, V] logits never exist in memory.
//
// Orientation.  The vocabulary is the M side of the MFMA tile and tokens are the N side: in the
// 32x32 result layout a lane then owns one token column and 16 vocabulary rows, so the log-sum-exp
// over the vocabulary is mostly a per-lane reduction; lanes are only combined once per sweep.
//
// Tiling.  A workgroup of 256 threads (4 wavefronts, one per SIMD) computes a 256 (vocabulary) x
// 256 (tokens) tile, each wavefront a 128 x 128 quarter = 4 x 4 MFMA tiles = 256 accumulator
// registers.  K (the hidden size) is walked in chunks of 64 through LDS, double buffered:
// global -> registers for chunk c+1 is issued before the MFMAs of chunk c.  LDS rows are padded
// from 128 to 144 bytes so that the 16-byte fragment reads of 16 consecutive rows hit distinct
// banks.
//
// Schedule.  256 persistent workgroups = 8 XCDs x 32.  Inside an XCD the 32 workgroups form a
// 4 (token tiles) x 8 (vocabulary tiles) block that moves through the vocabulary together, so at
// any time they share 4 hidden-state tiles and 8 weight tiles through that XCD's L2 instead of
// each pulling its own 64 KiB per chunk from HBM.  A workgroup keeps one token tile for a whole
// sweep over its vocabulary tiles (stride 8) and writes one partial (max, sum) per token at the
// end; a small kernel merges the 8 partials per token, adds the chosen logit (a separate dot
// product) and writes log pi.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

constexpr int kLmTile = 256;         // tile edge, both sides
constexpr int kLmChunk = 64;         // K elements per LDS stage
constexpr int kLmRowBytes = 144;     // 64 bf16 = 128 bytes + 16 bytes of padding
constexpr int kLmOperandBytes = kLmTile * kLmRowBytes;  // 36,864
constexpr int kLmLdsBytes = 4 * kLmOperandBytes;        // 2 stages x 2 operands = 147,456
constexpr int kLmThreads = 256;
constexpr int kLmVocabStrides = 8;   // vocabulary tiles walked with this stride (partials per token)
constexpr int kLmTokenTilesPerXcd = 4;

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t lm_u32x4_t __attribute__((ext_vector_type(4)));

// Folds the 64 vocabulary rows this lane holds of token column b (4 MFMA tiles x 16 values) into
// the lane's running (max, sum).  Row offset of acc[a][b][4 i + j] inside the lane's slice is
// a 32 + 8 i + j; offsets >= vlim lie past the vocabulary (only in the last, ragged tile).
// The accumulators are only read, never modified.
template <bool RAGGED>
__device__ __forceinline__ void fold_column(const f32x16_t (&acc)[4][4], int b, int vlim, float &run_m, float &run_s)
{
    float mx = -INFINITY;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float v = acc[a][b][e];
            if (RAGGED && a * 32 + (e >> 2) * 8 + (e & 3) >= vlim) v = -INFINITY;
            mx = fmaxf(mx, v);
        }
    const float m_new = fmaxf(run_m, mx);
    const float nm = -m_new * kLog2e;
    float s = run_s * exp2_hw((run_m - m_new) * kLog2e);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float v = acc[a][b][e];
            if (RAGGED && a * 32 + (e >> 2) * 8 + (e & 3) >= vlim) v = -INFINITY;
            s += exp2_hw(fmaf(v, kLog2e, nm));
        }
    run_m = m_new;
    run_s = s;
}

__global__ __launch_bounds__(kLmThreads) void lmhead_lse_kernel(const uint16_t *__restrict__ W,
                                                                const uint16_t *__restrict__ h, int64_t T, int64_t H,
                                                                int64_t V, float2 *__restrict__ partial)
{
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;          // vocabulary half, token half of the tile
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int mt = slot & (kLmTokenTilesPerXcd - 1), nt = slot / kLmTokenTilesPerXcd;
    const int ntt = (int)((T + kLmTile - 1) / kLmTile), nvt = (int)((V + kLmTile - 1) / kLmTile);
    const int ngroups = (ntt + kLmTokenTilesPerXcd - 1) / kLmTokenTilesPerXcd;
    const int nchunks = (int)(H / kLmChunk);

    // global -> LDS staging: thread owns the 16-byte piece `piece` of rows lrow + 32 j
    const int piece = tid & 7, lrow = tid >> 3;
    const uint32_t st_off = (uint32_t)lrow * kLmRowBytes + (uint32_t)piece * 16;
    // fragment reads: row (lane & 31) of an MFMA tile, k half (lane >> 5)
    const uint32_t fa_off = (uint32_t)(wm * 128 + (lane & 31)) * kLmRowBytes + (uint32_t)(lane >> 5) * 16;
    const uint32_t fb_off = (uint32_t)(wn * 128 + (lane & 31)) * kLmRowBytes + (uint32_t)(lane >> 5) * 16;

    for (int g = xcd; g < ngroups; g += 8) {
        const int tt = g * kLmTokenTilesPerXcd + mt;
        if (tt >= ntt) continue;  // uniform over the workgroup
        const int64_t t0 = (int64_t)tt * kLmTile;

        // per-thread element offsets of its 8 staging rows inside the token tile (clamped: tokens
        // past the end are computed but never written)
        const char *h_tile = reinterpret_cast<const char *>(h + t0 * H);
        const int t_last = (int)(T - 1 - t0);  // last valid row of this tile (>= 0)
        uint32_t boff[8];                      // byte offsets inside the tile (< 2^32: 256 rows x H x 2)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = min(lrow + 32 * j, t_last);
            boff[j] = (uint32_t)r * (uint32_t)H * 2u + (uint32_t)piece * 16u;
        }
        float run_m[4], run_s[4];
#pragma unroll
        for (int tn = 0; tn < 4; ++tn) {
            run_m[tn] = kNegFloor;
            run_s[tn] = 0.0f;
        }

        for (int vt = nt; vt < nvt; vt += kLmVocabStrides) {
            const int64_t v0 = (int64_t)vt * kLmTile;
            const char *w_tile = reinterpret_cast<const char *>(W + v0 * H);
            const int v_last = (int)(V - 1 - v0);
            uint32_t aoff[8];  // rows past the vocabulary are clamped here and masked below
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = min(lrow + 32 * j, v_last);
                aoff[j] = (uint32_t)r * (uint32_t)H * 2u + (uint32_t)piece * 16u;
            }
            f32x16_t acc[4][4];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

            // K loop, one barrier per chunk.  While the MFMAs of chunk c run from LDS buffer c & 1,
            // the chunk staged in registers (c+1) is written to the other buffer and the global
            // loads of chunk c+2 are issued into the registers just freed; LDS writes, global loads
            // and the fragment reads of the next k-step are interleaved with the MFMAs.  The barrier
            // at the end of iteration c publishes buffer (c+1) & 1 and guarantees that nobody still
            // reads buffer c & 1 when iteration c+1 overwrites it.  Past the last chunk the loads are
            // clamped to it (re-read) instead of branching.
            lm_u32x4_t ga[8], gb[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                ga[j] = *reinterpret_cast<const lm_u32x4_t *>(w_tile + aoff[j]);
                gb[j] = *reinterpret_cast<const lm_u32x4_t *>(h_tile + boff[j]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                *reinterpret_cast<lm_u32x4_t *>(lds + st_off + j * 32 * kLmRowBytes) = ga[j];
                *reinterpret_cast<lm_u32x4_t *>(lds + kLmOperandBytes + st_off + j * 32 * kLmRowBytes) = gb[j];
            }
            {
                const uint32_t koff = (uint32_t)min(1, nchunks - 1) * (kLmChunk * 2);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    ga[j] = *reinterpret_cast<const lm_u32x4_t *>(w_tile + (size_t)(aoff[j] + koff));
                    gb[j] = *reinterpret_cast<const lm_u32x4_t *>(h_tile + (size_t)(boff[j] + koff));
                }
            }
            __syncthreads();
#pragma unroll 1
            for (int c = 0; c < nchunks; ++c) {
                const char *sa = lds + (c & 1) * 2 * kLmOperandBytes;
                const char *sb = sa + kLmOperandBytes;
                char *da = lds + ((c + 1) & 1) * 2 * kLmOperandBytes;
                char *db = da + kLmOperandBytes;
                const uint32_t koff = (uint32_t)min(c + 2, nchunks - 1) * (kLmChunk * 2);
                bf16x8_t fa[2][4], fb[2][4];
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    fa[0][a] = *reinterpret_cast<const bf16x8_t *>(sa + fa_off + a * 32 * kLmRowBytes);
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    fb[0][b] = *reinterpret_cast<const bf16x8_t *>(sb + fb_off + b * 32 * kLmRowBytes);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    if (ks < 3) {
#pragma unroll
                        for (int a = 0; a < 4; ++a)
                            fa[(ks + 1) & 1][a] = *reinterpret_cast<const bf16x8_t *>(sa + fa_off + a * 32 * kLmRowBytes + (ks + 1) * 32);
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            fb[(ks + 1) & 1][b] = *reinterpret_cast<const bf16x8_t *>(sb + fb_off + b * 32 * kLmRowBytes + (ks + 1) * 32);
                    }
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const int j = 2 * ks + jj;
                        *reinterpret_cast<lm_u32x4_t *>(da + st_off + j * 32 * kLmRowBytes) = ga[j];
                        *reinterpret_cast<lm_u32x4_t *>(db + st_off + j * 32 * kLmRowBytes) = gb[j];
                        ga[j] = *reinterpret_cast<const lm_u32x4_t *>(w_tile + (size_t)(aoff[j] + koff));
                        gb[j] = *reinterpret_cast<const lm_u32x4_t *>(h_tile + (size_t)(boff[j] + koff));
                    }
#pragma unroll
                    for (int a = 0; a < 4; ++a)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][a], fb[ks & 1][b], acc[a][b], 0, 0, 0);
                    // spread this k-step's memory instructions between its MFMAs
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);  // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // LDS reads (next k-step's fragments)
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write (next chunk)
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global load (chunk after next)
                    }
                }
                __syncthreads();
            }

            // ---- fold the tile into the running (max, sum) of this lane's four token columns ----
            // acc[a][b][4 i + j] = z[vocab v0 + wm 128 + a 32 + 8 i + (lane >> 5) 4 + j][token column b]
            const bool ragged = v0 + kLmTile > V;  // last vocabulary tile: rows past V are masked
            const int vlim = (int)(V - v0) - wm * 128 - (lane >> 5) * 4;  // row offsets >= vlim are past V
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (ragged) fold_column<true>(acc, b, vlim, run_m[b], run_s[b]);
                else fold_column<false>(acc, b, vlim, run_m[b], run_s[b]);
                __builtin_amdgcn_sched_barrier(0);  // one token column at a time
            }
        }

        // ---- end of the sweep: merge the two lane halves, then the two vocabulary halves ----
        float2 *red = reinterpret_cast<float2 *>(lds);  // [2][256]; tile buffers are idle after the last barrier
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            MaxSum mine = {run_m[b], run_s[b]};
            MaxSum other = {__shfl_xor(mine.m, 32, kWave), __shfl_xor(mine.s, 32, kWave)};
            mine = combine(mine, other);
            if (lane < 32) red[wm * kLmTile + wn * 128 + b * 32 + lane] = make_float2(mine.m, mine.s);
        }
        __syncthreads();
        {
            const float2 p0 = red[tid], p1 = red[kLmTile + tid];
            const MaxSum tot = combine(MaxSum{p0.x, p0.y}, MaxSum{p1.x, p1.y});
            if (t0 + tid < T) partial[(int64_t)nt * T + t0 + tid] = make_float2(tot.m, tot.s);
        }
        __syncthreads();
    }
}

// z[t, y_t] = h[t, :] . W[y_t, :] in fp32, one wavefront per token; then
// lse_t from the kLmVocabStrides partials and log pi = z_y - lse.
__global__ __launch_bounds__(256) void lmhead_finish_kernel(const uint16_t *__restrict__ W,
                                                            const uint16_t *__restrict__ h, int64_t T, int64_t H,
                                                            int64_t V, const int32_t *__restrict__ chosen,
                                                            const float2 *__restrict__ partial, int nparts,
                                                            float *logp, float *lse_out)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
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
            const float2 q = partial[(int64_t)p * T + t];
            tot = combine(tot, MaxSum{q.x, q.y});
        }
        const float lse = tot.m + logf(tot.s);
        if (lse_out) lse_out[t] = lse;
        logp[t] = ok ? dot - lse : 0.0f;
    }
}

size_t lmhead_workspace_bytes(int64_t T)
{
    const size_t t = (size_t)(T > 0 ? T : 0);
    return ((t * kLmVocabStrides * sizeof(float2) + 255) / 256) * 256 + 256;
}

hipError_t launch_fused_lmhead_logprob(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                       const int32_t *chosen, float *logp, float *lse, void *workspace, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(lmhead_lse_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLmLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    float2 *partial = reinterpret_cast<float2 *>(workspace);
    hipLaunchKernelGGL(lmhead_lse_kernel, dim3(256), dim3(kLmThreads), kLmLdsBytes, s,
                       reinterpret_cast<const uint16_t *>(weight), reinterpret_cast<const uint16_t *>(hidden), T, H, V,
                       partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((T + 3) / 4);
    hipLaunchKernelGGL(lmhead_finish_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<const uint16_t *>(weight),
                       reinterpret_cast<const uint16_t *>(hidden), T, H, V, chosen, partial, kLmVocabStrides, logp, lse);
    return hipGetLastError();
}

}  // namespace a3po
