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
// registers.  K (the hidden size) is walked in stages of 32 through a ring of LDS buffers that
// direct global -> LDS loads fill a few stages ahead; the 16-byte pieces of a row are stored
// permuted so that fragment reads are free of bank conflicts without padding.
//
// Schedule.  256 persistent workgroups = 8 XCDs x 32.  Inside an XCD the 32 workgroups form a
// 4 (token tiles) x 8 (vocabulary tiles) block that moves through the vocabulary together, so at
// any time they share 4 hidden-state tiles and 8 weight tiles through that XCD's L2 instead of
// each pulling its own 32 KiB per stage from HBM.  A workgroup keeps one token tile for a whole
// sweep over its vocabulary tiles (stride 8) and writes one partial (max, sum) per token at the
// end; a small kernel merges the 8 partials per token, adds the chosen logit (a separate dot
// product) and writes log pi.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

constexpr int kLmTile = 256;         // tile edge, both sides
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
// The scheduling fences after each MFMA tile keep the copies of the accumulators short-lived: without
// them the register allocator spills across the K loop and a reload there waits for every direct load
// in flight.
template <bool RAGGED>
__device__ __forceinline__ void fold_column(const f32x16_t (&acc)[4][4], int b, int vlim, float &run_m, float &run_s)
{
    float mx = -INFINITY;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float v = acc[a][b][e];
            if (RAGGED && a * 32 + (e >> 2) * 8 + (e & 3) >= vlim) v = -INFINITY;
            mx = fmaxf(mx, v);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const float m_new = fmaxf(run_m, mx);
    float s = run_s * exp2_hw((run_m - m_new) * kLog2e);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float v = acc[a][b][e];
            if (RAGGED && a * 32 + (e >> 2) * 8 + (e & 3) >= vlim) v = -INFINITY;
            s += exp2_hw((v - m_new) * kLog2e);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    run_m = m_new;
    run_s = s;
}

// ---------------------------------------------------------------------------------------
// Operands reach LDS by direct global -> LDS loads (global_load_lds_dwordx4: lane l of a wavefront
// lands at lds_base + 16 l; no staging registers, no LDS write instructions), into a ring of
// kDmaStages stages of 32 K-elements each, with up to kDmaStages - 1 stages in flight.
//
// LDS layout of one operand stage: 256 rows x 64 bytes, unpadded (a direct load fills 16 rows x 64
// bytes contiguously).  The 16-byte piece p of row r is stored at physical piece p ^ ((r >> 2) & 3):
// the permutation is applied on the global side (each lane fetches the logical piece that belongs
// at its physical position), so a fragment read - 16 consecutive rows, same logical piece - touches
// 16 distinct bank groups.
//
// Schedule of stage i (two k-steps of 16 MFMAs).  A wavefront holds the fragments of a whole stage
// in registers, twice (this stage and the next).  At the top of stage i it waits for its own loads
// of stage i+1 and for its own fragment reads of stage i, and all wavefronts meet at one barrier:
// stage i+1 is now visible and the slot of stage i is free (everybody has it in registers).  During
// the 32 MFMAs of stage i the 16 fragments of stage i+1 are read and the 8 direct loads of stage
// i + kDmaStages are issued into the freed slot, two reads and one load per group of four MFMAs, so
// both streams are spread evenly over the stage.
constexpr int kDmaStages = 4;
constexpr int kDmaK = 32;                                  // K elements per stage
constexpr int kDmaRowBytes = kDmaK * 2;                    // 64
constexpr int kDmaOperandBytes = kLmTile * kDmaRowBytes;   // 16,384
constexpr int kDmaStageBytes = 2 * kDmaOperandBytes;       // 32,768
constexpr int kDmaLdsBytes = kDmaStages * kDmaStageBytes;  // 131,072 of the compute unit's 163,840

typedef __attribute__((address_space(3))) void *lds_ptr_t;

__device__ __forceinline__ void dma16(const char *g, char *l)
{
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const lm_u32x4_t *>(g), (lds_ptr_t)l, 16, 0, 0);
}

// QUAD: the hidden size is a multiple of kDmaStages stages.  Then every tile starts in ring slot 0,
// the K loop is unrolled by the ring depth (all LDS addresses are constants) and the refill cursor
// moves once per kDmaStages stages.  Otherwise the loop is unrolled by two (the fragment buffers
// alternate; the number of stages is even) and slot and cursor are tracked per stage.
template <bool QUAD>
__global__ __launch_bounds__(kLmThreads) void lmhead_lse_kernel(const uint16_t *__restrict__ W,
                                                                    const uint16_t *__restrict__ h, int64_t T,
                                                                    int64_t H, int64_t V, float2 *__restrict__ partial)
{
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;          // vocabulary half, token half of the tile
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int mt = slot & (kLmTokenTilesPerXcd - 1), nt = slot / kLmTokenTilesPerXcd;
    const int ntt = (int)((T + kLmTile - 1) / kLmTile), nvt = (int)((V + kLmTile - 1) / kLmTile);
    const int ngroups = (ntt + kLmTokenTilesPerXcd - 1) / kLmTokenTilesPerXcd;
    const int nstages = (int)(H / kDmaK);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);  // the wavefront number in a scalar register

    // direct loads: instruction j of an operand covers tile rows (4 j + wave) 16 .. + 15; lane -> row lane >> 2,
    // physical piece lane & 3, which holds logical piece (lane & 3) ^ ((row >> 2) & 3) = (lane & 3) ^ ((lane >> 4) & 3)
    const int drow = lane >> 2;
    const uint32_t dpiece = (uint32_t)((lane & 3) ^ ((lane >> 4) & 3)) * 16u;
    // fragment reads: row lane & 31 of a 32-row MFMA tile, k half lane >> 5 of k-step s: logical piece 2 s + (lane >> 5),
    // physical piece that ^ ((row >> 2) & 3) = that ^ ((lane >> 2) & 3)
    const uint32_t fr[2] = {(uint32_t)(lane & 31) * kDmaRowBytes + (uint32_t)(((lane >> 5) ^ ((lane >> 2) & 3)) * 16),
                            (uint32_t)(lane & 31) * kDmaRowBytes + (uint32_t)(((2 + (lane >> 5)) ^ ((lane >> 2) & 3)) * 16)};
    const uint32_t fa_base = (uint32_t)(wm * 128) * kDmaRowBytes;
    const uint32_t fb_base = kDmaOperandBytes + (uint32_t)(wn * 128) * kDmaRowBytes;

    for (int g = xcd; g < ngroups; g += 8) {
        const int tt = g * kLmTokenTilesPerXcd + mt;
        if (tt >= ntt) continue;  // uniform over the workgroup
        const int64_t t0 = (int64_t)tt * kLmTile;
        const char *h_tile = reinterpret_cast<const char *>(h + t0 * H);
        const int t_last = (int)(T - 1 - t0);
        uint32_t boff[4];  // rows past the end are clamped (computed, never written)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            boff[j] = (uint32_t)min((4 * j + wave) * 16 + drow, t_last) * (uint32_t)H * 2u + dpiece;
        float run_m[4], run_s[4];
#pragma unroll
        for (int tn = 0; tn < 4; ++tn) {
            run_m[tn] = kNegFloor;
            run_s[tn] = 0.0f;
        }

        // The ring runs through the whole sweep without a break: the refills of a tile's last stages already
        // bring the next tile's first stages, so a tile's fold epilogue overlaps with their arrival and there
        // is one prologue and one drain per sweep.  The refill cursor (r_*) names the stage the next refill
        // loads (QUAD: the first of a group of kDmaStages stages); past the workgroup's last tile it stays on
        // that tile's last stage (group): reloads of bytes that are already there, which keep the number of
        // loads per stage, and with it the s_waitcnt arithmetic, constant.
        if (nt < nvt) {  // uniform over the workgroup
            const int last_vt = nt + ((nvt - 1 - nt) / kLmVocabStrides) * kLmVocabStrides;
            // weight-row offsets; in the vocabulary's last tile rows past V are clamped
            uint32_t aoff_last[4], aoff[4];
            const int v_last_global = (int)(V - 1 - (int64_t)(nvt - 1) * kLmTile);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = (4 * j + wave) * 16 + drow;
                aoff_last[j] = (uint32_t)min(r, v_last_global) * (uint32_t)H * 2u + dpiece;
                aoff[j] = nt == nvt - 1 ? aoff_last[j] : (uint32_t)r * (uint32_t)H * 2u + dpiece;
            }
            int r_vt = nt, r_k = 0;
            const char *r_w = reinterpret_cast<const char *>(W + (int64_t)r_vt * kLmTile * H);
            // direct load number q of one operand (0: weight rows, 1: hidden rows) of stage r_k + u into ring slot sl
            auto refill = [&](int sl, int q, int u, int operand) {
                const uint32_t koff = (uint32_t)(r_k + u) * (uint32_t)kDmaRowBytes;
                char *dst = lds + sl * kDmaStageBytes + wave_s * 1024 + q * 4096;
                if (operand == 0) dma16(r_w + koff + aoff[q], dst);
                else dma16(h_tile + koff + boff[q], dst + kDmaOperandBytes);
            };
            auto advance = [&](int step) {
                if (r_k + step < nstages) {
                    r_k += step;
                } else if (r_vt < last_vt) {
                    r_k = 0;
                    r_vt += kLmVocabStrides;
                    r_w = reinterpret_cast<const char *>(W + (int64_t)r_vt * kLmTile * H);
                    if (r_vt == nvt - 1) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) aoff[j] = aoff_last[j];
                    }
                }
            };

            // prologue: fill the whole ring, then wait for the first stage and read its fragments
#pragma unroll
            for (int st = 0; st < kDmaStages; ++st) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    refill(st, q, QUAD ? st : 0, 0);
                    refill(st, q, QUAD ? st : 0, 1);
                }
                if (!QUAD) advance(1);
            }
            if (QUAD) advance(kDmaStages);
            {
                constexpr int kAllow = 8 * (kDmaStages - 1);  // everything issued after the first stage
                __builtin_amdgcn_s_waitcnt(0x0F70 | (kAllow & 15) | ((kAllow >> 4) << 14));
            }
            __builtin_amdgcn_s_barrier();  // bare, as in the K loop: the rest of the ring stays in flight
            bf16x8_t fa[2][2][4], fb[2][2][4];  // [buffer][k-step][MFMA tile]
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    fa[0][ks][a] = *reinterpret_cast<const bf16x8_t *>(lds + fa_base + a * 32 * kDmaRowBytes + fr[ks]);
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    fb[0][ks][b] = *reinterpret_cast<const bf16x8_t *>(lds + fb_base + b * 32 * kDmaRowBytes + fr[ks]);
            }
            int sl_dyn = 0;  // ring slot of the stage being computed (tracked only when !QUAD)

            for (int vt = nt; vt < nvt; vt += kLmVocabStrides) {
                const int64_t v0 = (int64_t)vt * kLmTile;
                f32x16_t acc[4][4];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

                // One stage out of the fragments in buffer p (read from ring slot sl during the stage before);
                // u: the stage's position in the cursor's group (0 when !QUAD).
                auto stage = [&](const int sl, const int u, const int p) __attribute__((always_inline)) {
                    const int nsl = sl + 1 == kDmaStages ? 0 : sl + 1;
                    const char *nxt = lds + nsl * kDmaStageBytes;
                    __builtin_amdgcn_sched_barrier(0);
                    // The next stage has landed (own loads: the kDmaStages - 2 stages after it may still be in
                    // flight) and this stage is in registers (own reads, lgkmcnt(0)): meet.  A bare barrier: the
                    // fence that __syncthreads() carries makes the compiler drain every direct load it can see in
                    // flight (vmcnt(0)), which would empty the ring at each stage.
                    __builtin_amdgcn_s_waitcnt(0x0070 | (8 * (kDmaStages - 2) & 15) | ((8 * (kDmaStages - 2) >> 4) << 14));
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int grp = 0; grp < 8; ++grp) {   // k-step grp >> 2, vocabulary MFMA tile grp & 3
                        const int ks = grp >> 2, q = grp & 3;
                        // two fragments of the next stage (the next tile's first stage, at the end of a tile) ...
                        if (q < 2) {
#pragma unroll
                            for (int a = 2 * q; a < 2 * q + 2; ++a)
                                fa[p ^ 1][ks][a] = *reinterpret_cast<const bf16x8_t *>(nxt + fa_base + a * 32 * kDmaRowBytes + fr[ks]);
                        } else {
#pragma unroll
                            for (int b = 2 * q - 4; b < 2 * q - 2; ++b)
                                fb[p ^ 1][ks][b] = *reinterpret_cast<const bf16x8_t *>(nxt + fb_base + b * 32 * kDmaRowBytes + fr[ks]);
                        }
                        // ... one direct load into the slot this stage came from ...
                        refill(sl, grp >> 1, u, grp & 1);
                        // ... and four MFMAs
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[q][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[p][ks][q], fb[p][ks][b], acc[q][b], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };
                if (QUAD) {
                    static_assert(kDmaStages == 4, "the unrolled loop names the four ring slots");
#pragma unroll 1
                    for (int i = 0; i < nstages; i += kDmaStages) {
                        stage(0, 0, 0);
                        stage(1, 1, 1);
                        stage(2, 2, 0);
                        stage(3, 3, 1);
                        advance(kDmaStages);
                    }
                } else {
#pragma unroll 1
                    for (int i = 0; i < nstages; i += 2) {  // H % 64 == 0: an even number of stages
                        stage(sl_dyn, 0, 0);
                        advance(1);
                        sl_dyn = sl_dyn + 1 == kDmaStages ? 0 : sl_dyn + 1;
                        stage(sl_dyn, 0, 1);
                        advance(1);
                        sl_dyn = sl_dyn + 1 == kDmaStages ? 0 : sl_dyn + 1;
                    }
                }

                // ---- fold the tile into the running (max, sum) of this lane's four token columns, while the
                // next tile's first stages arrive ----
                const bool ragged = v0 + kLmTile > V;
                const int vlim = (int)(V - v0) - wm * 128 - (lane >> 5) * 4;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (ragged) fold_column<true>(acc, b, vlim, run_m[b], run_s[b]);
                    else fold_column<false>(acc, b, vlim, run_m[b], run_s[b]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // drain: the reloads past the last stage must have landed before the ring's memory is reused
            __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
            __syncthreads();
        }

        // ---- end of the sweep: merge the two lane halves, then the two vocabulary halves ----
        float2 *red = reinterpret_cast<float2 *>(lds);  // [2][256]; the ring is idle after the drain barrier
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
        const float log_s = logf(tot.s);
        if (lse_out) lse_out[t] = tot.m + log_s;
        logp[t] = ok ? (dot - tot.m) - log_s : 0.0f;
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
    const bool quad = H % (kDmaK * kDmaStages) == 0;
    auto *kernel = quad ? lmhead_lse_kernel<true> : lmhead_lse_kernel<false>;
    static bool attr_set[2] = {false, false};
    if (!attr_set[quad]) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLdsBytes);
        if (e != hipSuccess) return e;
        attr_set[quad] = true;
    }
    float2 *partial = reinterpret_cast<float2 *>(workspace);
    hipLaunchKernelGGL(kernel, dim3(256), dim3(kLmThreads), kDmaLdsBytes, s,
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
