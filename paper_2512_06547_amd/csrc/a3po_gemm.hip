// bfloat16 contraction on the matrix cores for the LM-head path:  C[M, N] = A[M, K] B[N, K]^T, both operands
// row-major with the contracted index contiguous, fp32 accumulation (v_mfma_f32_16x16x32_bf16), and one of four
// epilogues applied to each 256 x 256 tile as it leaves the accumulators:
//   kEpiLse        fold the tile into a running (max, sum) per column n over the rows m (the online log-sum-exp
//                  of the vocabulary when A is the LM-head weight and B the hidden states); C is not written
//   kEpiLseStore   the same, and the tile is also stored as fp32 (the logits of a token chunk, kept for the
//                  backward pass)
//   kEpiStoreBf16  the tile is stored as bfloat16 (the gradient of the hidden states)
//   kEpiAccumF32   the tile is stored as fp32, or added to what C holds (the weight gradient, summed over chunks)
//
// Tiling.  A workgroup of 512 threads (8 wavefronts, two per SIMD) computes a 256 x 256 tile, each wavefront a
// 128 x 64 part = 8 x 4 MFMA tiles of 16 x 16 = 128 accumulator registers.  Two wavefronts per SIMD: while one
// waits (for the stage barrier, for its fragments) the other keeps the matrix core busy, which one wavefront with
// 256 accumulators cannot; the 16 x 16 x 32 instruction also draws less power per flop than the 32 x 32 x 16 one,
// and at these sizes the chip is power-limited (the clock falls as the matrix cores get busier).  In the 16 x 16
// result layout a lane owns one column n and 4 rows m of each MFMA tile, so a reduction over m is mostly per
// lane.
//
// K is walked in stages of 32 (one MFMA deep) through a ring of LDS buffers that direct global -> LDS loads
// (global_load_lds_dwordx4: lane l of a wavefront lands at lds_base + 16 l; no staging registers, no LDS write
// instructions) fill a few stages ahead.  LDS layout of one operand stage: 256 rows x 64 bytes, unpadded; the
// 16-byte piece p of row r sits at physical piece p ^ ((r >> 2) & 3) - the permutation is applied on the global
// side of the load - so a fragment read (16 consecutive rows, same logical piece) touches 16 distinct bank groups.
//
// Schedule of stage i (32 MFMAs per wavefront).  At the top a wavefront waits for its own loads of stage i+1 and
// its own fragment reads, and all wavefronts meet at one barrier: stage i+1 is now visible and the slot of stage i
// is free.  The 8 row fragments live in one set of registers: each is re-read for stage i+1 right after its last
// use in stage i; the 4 column fragments, which every MFMA group of the stage needs, alternate between two sets.
// The 4 direct loads of stage i + kDmaStages go into the freed slot, spread over the stage.  The ring runs through
// a workgroup's whole sequence of tiles without a break: the refills of a tile's last stages already bring the
// next tile's first stages, so a tile's epilogue overlaps with their arrival.
//
// Tile order.  One persistent workgroup per compute unit; the workgroups of an XCD (dispatch order deals
// workgroups round-robin over the XCDs) form a block of ml_count x 4 tiles that share ml_count tiles of A and 4
// tiles of B through that XCD's L2.  The tile grid is cut into such blocks ("pairs" of a 4-tile column group and an
// ml_count-tile row round); pair p = group * rounds + round, and each XCD takes a contiguous range of pairs, i.e.
// it sweeps down the rows of one column group before it moves to the next.  With kEpiLse* a workgroup therefore
// keeps its running (max, sum) in registers over a whole sweep and writes one partial per column per sweep.
//
// Operand and result layouts.  An operand is either row-major (row stride lda / ldb) or in panels of 256 rows x 32
// contracted elements (a3po_launch.h), in which the 16 rows x 64 bytes of a direct load are 1 KiB of contiguous
// memory.  The fp32 epilogues can store the tile transposed (element (m, n) at C[n ldc + m]): a lane's four
// accumulator values of one MFMA tile are four consecutive m of one n, i.e. one 16-byte store without staging.
// One of M, N, K may be known only on the device (DynCount): the launch is sized for the host's upper bound and
// every workgroup reads the extent first; beyond it there is nothing to do and it returns.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

constexpr int kGemmTile = 256;  // tile edge, both sides
constexpr int kGemmThreads = 512;
constexpr int kGemmWaves = kGemmThreads / kWave;
constexpr int kGemmColTiles = 4;  // tiles of B (columns) side by side in an XCD's block

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t gemm_u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kDmaStages = 4;
constexpr int kDmaK = 32;                                  // K elements per stage
constexpr int kDmaRowBytes = kDmaK * 2;                    // 64
constexpr int kDmaOperandBytes = kGemmTile * kDmaRowBytes; // 16,384
constexpr int kDmaStageBytes = 2 * kDmaOperandBytes;       // 32,768
constexpr int kDmaRingBytes = kDmaStages * kDmaStageBytes; // 131,072 of the compute unit's 163,840
constexpr int kGemmRedBytes = 2 * kGemmTile * (int)sizeof(float2);  // column partials of the two row halves
// per-wavefront staging tile of the store epilogues: 16 rows x 32 columns of fp32, rows 36 floats apart
constexpr int kStageLd = 36;
constexpr int kStageBytes = 16 * kStageLd * (int)sizeof(float);  // 2,304
constexpr int kGemmLdsBytes = kDmaRingBytes + kGemmRedBytes + kGemmWaves * kStageBytes;  // 153,600 of 163,840

typedef __attribute__((address_space(3))) void *lds_ptr_t;

__device__ __forceinline__ void dma16(const char *g, char *l)
{
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const gemm_u32x4_t *>(g), (lds_ptr_t)l, 16, 0, 0);
}

// s_waitcnt with the given vector-memory and LDS counts (the export count is left alone)
__device__ __forceinline__ constexpr int waitcnt_imm(int vmcnt, int lgkmcnt)
{
    return 0x0070 | (vmcnt & 15) | ((vmcnt >> 4) << 14) | ((lgkmcnt & 15) << 8);
}
constexpr int kNoVmWait = 63, kNoLgkmWait = 15;

// Accumulator layout of a wavefront: acc[a][b][i] is row a 16 + 4 (lane >> 4) + i, column b 16 + (lane & 15) of its
// 128 x 64 part of the tile.

// Folds the 32 rows this lane holds of column block b (8 MFMA tiles x 4 values) into the lane's running
// (max, sum).  Row offsets >= mlim lie past the last row (only in the last, ragged tile); mlim is relative to the
// lane's first row.  The accumulators are only read.
template <bool RAGGED>
__device__ __forceinline__ void fold_column(const f32x4_t (&acc)[8][4], int b, int mlim, float &run_m, float &run_s)
{
    float mx = -INFINITY;
#pragma unroll
    for (int a = 0; a < 8; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = acc[a][b][i];
            if (RAGGED && a * 16 + i >= mlim) v = -INFINITY;
            mx = fmaxf(mx, v);
        }
    }
    const float m_new = fmaxf(run_m, mx);
    float s = run_s * exp2_hw((run_m - m_new) * kLog2e);
#pragma unroll
    for (int a = 0; a < 8; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = acc[a][b][i];
            if (RAGGED && a * 16 + i >= mlim) v = -INFINITY;
            s += exp2_hw((v - m_new) * kLog2e);
        }
    }
    run_m = m_new;
    run_s = s;
}

// Element-wise store of a wavefront's part of the tile: one accumulator register covers 4 rows x 16 consecutive
// columns.  EDGE: the tile reaches past M or N; rows / columns beyond are skipped.  Used for tiles on the edge and
// for sums into C, which go through the memory side's adders (every element has one owner per launch and launches
// are ordered on the stream, so the sum is deterministic; nobody waits for its result).
template <int EPI, bool EDGE>
__device__ __forceinline__ void store_tile(const f32x4_t (&acc)[8][4], void *C, int64_t ldc, int64_t m0, int64_t n0,
                                           int64_t M, int64_t N, int wm, int wn, int lane, bool add)
{
    const int col0 = wn * 64 + (lane & 15);
    const int row0 = wm * 128 + 4 * (lane >> 4);
    const int rows_left = (int)(M - m0 < kGemmTile ? M - m0 : kGemmTile);
    const int cols_left = (int)(N - n0 < kGemmTile ? N - n0 : kGemmTile);
#pragma unroll
    for (int a = 0; a < 8; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = row0 + a * 16 + i;
            if (EDGE && row >= rows_left) continue;
            const int64_t at = (m0 + row) * ldc + n0 + col0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (EDGE && col0 + b * 16 >= cols_left) continue;
                const float v = acc[a][b][i];
                if constexpr (EPI == kEpiStoreBf16) {
                    reinterpret_cast<uint16_t *>(C)[at + b * 16] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xFFFFu);
                } else if constexpr (EPI == kEpiAccumF32) {
                    float *p = reinterpret_cast<float *>(C) + at + b * 16;
                    if (add) unsafeAtomicAdd(p, v);
                    else *p = v;
                } else {
                    reinterpret_cast<float *>(C)[at + b * 16] = v;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// fp32 store of C^T (element (m, n) at C[n * ldc + m]): the four values of an accumulator register are four
// consecutive m of one column n, i.e. 16 contiguous bytes, so every register leaves with one 16-byte store and no
// staging; a wavefront's instruction covers 16 columns x 64 contiguous bytes.  M is a multiple of 4, so a group of
// four rows lies inside or outside as a whole.  `add`: sums into C through the memory side's adders.
template <bool EDGE>
__device__ __forceinline__ void store_tile_transposed(const f32x4_t (&acc)[8][4], float *C, int64_t ldc, int64_t m0,
                                                      int64_t n0, int64_t M, int64_t N, int wm, int wn, int lane, bool add)
{
    const int col0 = wn * 64 + (lane & 15);
    const int row0 = wm * 128 + 4 * (lane >> 4);
    const int rows_left = (int)(M - m0 < kGemmTile ? M - m0 : kGemmTile);
    const int cols_left = (int)(N - n0 < kGemmTile ? N - n0 : kGemmTile);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (EDGE && col0 + b * 16 >= cols_left) continue;
        float *col = C + (n0 + col0 + b * 16) * ldc + m0 + row0;
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            if (EDGE && row0 + a * 16 >= rows_left) continue;
            if (add) {
#pragma unroll
                for (int i = 0; i < 4; ++i) unsafeAtomicAdd(col + a * 16 + i, acc[a][b][i]);
            } else {
                *reinterpret_cast<float4 *>(col + a * 16) = make_float4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The transposed store in bfloat16: the four values of a register are rounded and leave as one 8-byte store.
template <bool EDGE>
__device__ __forceinline__ void store_tile_transposed_bf16(const f32x4_t (&acc)[8][4], uint16_t *C, int64_t ldc, int64_t m0,
                                                           int64_t n0, int64_t M, int64_t N, int wm, int wn, int lane)
{
    const int col0 = wn * 64 + (lane & 15);
    const int row0 = wm * 128 + 4 * (lane >> 4);
    const int rows_left = (int)(M - m0 < kGemmTile ? M - m0 : kGemmTile);
    const int cols_left = (int)(N - n0 < kGemmTile ? N - n0 : kGemmTile);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (EDGE && col0 + b * 16 >= cols_left) continue;
        uint16_t *col = C + (n0 + col0 + b * 16) * ldc + m0 + row0;
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            if (EDGE && row0 + a * 16 >= rows_left) continue;
            *reinterpret_cast<uint2 *>(col + a * 16) =
                make_uint2(pack_bf16x2(acc[a][b][0], acc[a][b][1]), pack_bf16x2(acc[a][b][2], acc[a][b][3]));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The same for a tile that lies inside C, with 16-byte stores: 16 rows x 32 columns at a time go through a staging
// tile in LDS that belongs to this wavefront alone (LDS instructions of one wavefront execute in order, so no waits
// or barriers are needed between its writes and its reads) and leave as 8 rows x 128 bytes (fp32) or 8 rows x 64
// bytes (bfloat16) per store instruction.
template <int EPI>
__device__ __forceinline__ void store_tile_wide(const f32x4_t (&acc)[8][4], void *C, int64_t ldc, int64_t m0, int64_t n0,
                                                int wm, int wn, int lane, float *stage)
{
    static_assert(EPI == kEpiStoreBf16 || EPI == kEpiLseStore || EPI == kEpiAccumF32, "plain stores only");
    const int wcol = lane & 15, wrow = 4 * (lane >> 4);  // where this lane's accumulator registers sit in a 16 x 16 tile
    const int rrow = lane >> 3, rcol = (lane & 7) * 4;   // what it reads back: 4 consecutive columns of row rrow + 8 pass
#pragma unroll
    for (int a = 0; a < 8; ++a) {
#pragma unroll
        for (int bp = 0; bp < 2; ++bp) {  // column blocks 2 bp, 2 bp + 1
#pragma unroll
            for (int bb = 0; bb < 2; ++bb)
#pragma unroll
                for (int i = 0; i < 4; ++i) stage[(wrow + i) * kStageLd + bb * 16 + wcol] = acc[a][2 * bp + bb][i];
            asm volatile("" ::: "memory");
            const int64_t at = (m0 + wm * 128 + a * 16 + rrow) * ldc + n0 + wn * 64 + bp * 32 + rcol;
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const float4 v = *reinterpret_cast<const float4 *>(stage + (rrow + 8 * pass) * kStageLd + rcol);
                if constexpr (EPI == kEpiStoreBf16) {
                    *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(C) + at + (int64_t)pass * 8 * ldc) =
                        make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
                } else {
                    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(C) + at + (int64_t)pass * 8 * ldc) = v;
                }
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// QUAD: K is a multiple of kDmaStages stages.  Then every tile starts in ring slot 0, the K loop is unrolled by
// the ring depth (all LDS addresses are constants) and the refill cursor moves once per kDmaStages stages.
// Otherwise the loop is unrolled by two (the column fragments alternate; the number of stages is even) and slot
// and cursor are tracked per stage.
template <int EPI, bool QUAD>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_kernel(const GemmArgs g)
{
    extern __shared__ __align__(16) char lds[];
    constexpr bool LSE = EPI == kEpiLse || EPI == kEpiLseStore;
    constexpr int kLoads = 4;  // direct loads per wavefront and stage: two 16-row blocks of A, two of B
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;  // row half (128 rows), column quarter (64 columns) of the tile
    const int xcd = (int)(blockIdx.x % (unsigned)g.nxcd), slot = (int)(blockIdx.x / (unsigned)g.nxcd);
    const int nl = slot & (kGemmColTiles - 1), ml = slot / kGemmColTiles;
    int64_t M = g.M, N = g.N, K = g.K;
    if (g.dyn_dim != kDynNone) {  // an extent that only the device knows (uniform: one scalar load)
        const int64_t v = dyn_extent(g.dyn, 0);
        if (g.dyn_dim == kDynM) M = v;
        else if (g.dyn_dim == kDynN) N = v;
        else K = (v + 127) / 128 * 128;
        if (v <= 0) return;
    }
    const int mtiles = (int)((M + kGemmTile - 1) / kGemmTile), ntiles = (int)((N + kGemmTile - 1) / kGemmTile);
    const int groups = (ntiles + kGemmColTiles - 1) / kGemmColTiles;
    const int rounds = (mtiles + g.ml_count - 1) / g.ml_count;
    const int64_t pairs = (int64_t)groups * rounds;
    const int64_t p_end = (int64_t)(xcd + 1) * pairs / g.nxcd;
    const int nstages = (int)(K / kDmaK);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);  // the wavefront number in a scalar register
    const uint32_t lda2 = (uint32_t)g.lda * 2u, ldb2 = (uint32_t)g.ldb * 2u;  // row strides in bytes

    // the first pair >= p in this XCD's range whose tile exists for this workgroup's place in the block (else p_end)
    auto next_tile = [&](int64_t p) {
        for (; p < p_end; ++p) {
            const int grp = (int)(p / rounds), rnd = (int)(p % rounds);
            if (rnd * g.ml_count + ml < mtiles && grp * kGemmColTiles + nl < ntiles) break;
        }
        return p;
    };

    // direct loads: instruction j of an operand covers tile rows (8 j + wave) 16 .. + 15; lane -> row lane >> 2,
    // physical piece lane & 3, which holds logical piece (lane & 3) ^ ((row >> 2) & 3) = (lane & 3) ^ ((lane >> 4) & 3)
    const int drow = lane >> 2;
    const uint32_t dpiece = (uint32_t)((lane & 3) ^ ((lane >> 4) & 3)) * 16u;
    // fragment reads: row lane & 15 of a 16-row block, k quarter lane >> 4 = logical piece, physical piece
    // that ^ ((row >> 2) & 3) = that ^ ((lane >> 2) & 3); block t of an operand starts at t * 1024 bytes
    const uint32_t fr = (uint32_t)(lane & 15) * kDmaRowBytes + (uint32_t)(((lane >> 4) ^ ((lane >> 2) & 3)) * 16);
    const uint32_t fa_base = (uint32_t)(wm * 8) * 1024u + fr;
    const uint32_t fb_base = kDmaOperandBytes + (uint32_t)(wn * 4) * 1024u + fr;

    int64_t p_cur = next_tile((int64_t)xcd * pairs / g.nxcd);
    if (p_cur >= p_end) return;  // uniform over the workgroup

    // The refill cursor names the tile (r_p) and stage (r_k; QUAD: the first of a group of kDmaStages stages) that
    // the next refill loads.  Past the workgroup's last tile it stays on that tile's last stage (group): reloads of
    // bytes that are already there, which keep the number of loads per stage, and with it the s_waitcnt
    // arithmetic, constant.  Rows past the end of an operand are clamped (computed, never written).
    int64_t r_p = p_cur;
    int r_k = 0;
    const char *r_a = nullptr, *r_b = nullptr;
    uint32_t aoff[2], boff[2];
    auto set_tile = [&](int64_t p) {
        const int mt = (int)(p % rounds) * g.ml_count + ml, nt = (int)(p / rounds) * kGemmColTiles + nl;
        r_a = reinterpret_cast<const char *>(g.A + (int64_t)mt * kGemmTile * g.lda);  // (a 256-row band of panels is as long)
        r_b = reinterpret_cast<const char *>(g.B + (int64_t)nt * kGemmTile * g.ldb);
        const int m_last = (int)(M - 1 - (int64_t)mt * kGemmTile), n_last = (int)(N - 1 - (int64_t)nt * kGemmTile);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = (8 * j + wave) * 16 + drow;
            // panels: every row of the band exists (padding), rows are 64 bytes apart
            aoff[j] = g.a_panel ? (uint32_t)r * 64u + dpiece : (uint32_t)min(r, m_last) * lda2 + dpiece;
            boff[j] = g.b_panel ? (uint32_t)r * 64u + dpiece : (uint32_t)min(r, n_last) * ldb2 + dpiece;
        }
    };
    set_tile(r_p);
    // direct load number q of one operand (0: A rows, 1: B rows) of stage r_k + u into ring slot sl
    auto refill = [&](int sl, int q, int u, int operand) {
        const uint32_t st = (uint32_t)(r_k + u);
        const uint32_t koff = st * (uint32_t)kDmaRowBytes;                 // rows: 64 bytes further along the row
        const uint32_t poff = st * 16384u;                                 // panels: the next block
        char *dst = lds + sl * kDmaStageBytes + wave_s * 1024 + q * 8192;
        if (operand == 0) dma16(r_a + (g.a_panel ? poff : koff) + aoff[q], dst);
        else dma16(r_b + (g.b_panel ? poff : koff) + boff[q], dst + kDmaOperandBytes);
    };
    auto advance = [&](int step) {
        if (r_k + step < nstages) {
            r_k += step;
        } else {
            const int64_t np = next_tile(r_p + 1);
            if (np < p_end) {
                r_p = np;
                r_k = 0;
                set_tile(np);
            }
        }
    };

    // prologue: fill the whole ring, then wait for the first stage and read its fragments
#pragma unroll
    for (int st = 0; st < kDmaStages; ++st) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            refill(st, q, QUAD ? st : 0, 0);
            refill(st, q, QUAD ? st : 0, 1);
        }
        if (!QUAD) advance(1);
    }
    if (QUAD) advance(kDmaStages);
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(kLoads * (kDmaStages - 1), kNoLgkmWait));  // everything issued after the first stage may fly
    __builtin_amdgcn_s_barrier();  // bare, as in the K loop: the rest of the ring stays in flight
    bf16x8_t fa[8], fb[2][4];
#pragma unroll
    for (int a = 0; a < 8; ++a) fa[a] = *reinterpret_cast<const bf16x8_t *>(lds + fa_base + a * 1024);
#pragma unroll
    for (int b = 0; b < 4; ++b) fb[0][b] = *reinterpret_cast<const bf16x8_t *>(lds + fb_base + b * 1024);
    int sl_dyn = 0;  // ring slot of the stage being computed (tracked only when !QUAD)

    float run_m[4], run_s[4];  // kEpiLse*: this lane's four columns over the sweep
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        run_m[b] = kNegFloor;
        run_s[b] = 0.0f;
    }

    while (p_cur < p_end) {
        const int grp = (int)(p_cur / rounds);
        const int64_t m0 = ((int64_t)(p_cur % rounds) * g.ml_count + ml) * kGemmTile;
        const int64_t n0 = ((int64_t)grp * kGemmColTiles + nl) * kGemmTile;
        f32x4_t acc[8][4];
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[a][b][i] = 0.0f;

        // One stage out of the row fragments fa and the column fragments fb[p] (read from ring slot sl during the
        // stage before); u: the stage's position in the cursor's group (0 when !QUAD).
        auto stage = [&](const int sl, const int u, const int p) __attribute__((always_inline)) {
            const int nsl = sl + 1 == kDmaStages ? 0 : sl + 1;
            const char *nxt = lds + nsl * kDmaStageBytes;
            __builtin_amdgcn_sched_barrier(0);
            // The next stage has landed (own loads: the kDmaStages - 2 stages after it may still be in flight) and
            // this stage is in registers (own reads, lgkmcnt(0)): meet.  A bare barrier: the fence that
            // __syncthreads() carries makes the compiler drain every direct load it can see in flight
            // (vmcnt(0)), which would empty the ring at each stage.
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(kLoads * (kDmaStages - 2), 0));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                // a column fragment of the next stage, a direct load into the slot this stage came from ...
                if (a < 4) fb[p ^ 1][a] = *reinterpret_cast<const bf16x8_t *>(nxt + fb_base + a * 1024);
                if ((a & 1) == 0) refill(sl, a >> 2, u, (a >> 1) & 1);
                // ... four MFMAs ...
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[a], fb[p][b], acc[a][b], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                // ... and this row fragment's successor, into the registers those MFMAs have just read
                fa[a] = *reinterpret_cast<const bf16x8_t *>(nxt + fa_base + a * 1024);
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
            for (int i = 0; i < nstages; i += 2) {  // K % 64 == 0: an even number of stages
                stage(sl_dyn, 0, 0);
                advance(1);
                sl_dyn = sl_dyn + 1 == kDmaStages ? 0 : sl_dyn + 1;
                stage(sl_dyn, 0, 1);
                advance(1);
                sl_dyn = sl_dyn + 1 == kDmaStages ? 0 : sl_dyn + 1;
            }
        }

        // ---- the tile's epilogue, while the next tile's first stages arrive ----
        const int64_t p_next = next_tile(p_cur + 1);
        const bool edge = m0 + kGemmTile > M || n0 + kGemmTile > N;  // uniform
        if constexpr (EPI != kEpiLse) {
            // tiles inside C leave with 16-byte stores (the launcher checks that rows of C start on 16 bytes);
            // only sums into C go element by element, through the memory side's adders
            float *stage_tile = reinterpret_cast<float *>(lds + kDmaRingBytes + kGemmRedBytes + wave_s * kStageBytes);
            if (EPI == kEpiStoreBf16 && g.transposed != 0) {
                uint16_t *ct = reinterpret_cast<uint16_t *>(g.C);
                if (edge) store_tile_transposed_bf16<true>(acc, ct, g.ldc, m0, n0, M, N, wm, wn, lane);
                else store_tile_transposed_bf16<false>(acc, ct, g.ldc, m0, n0, M, N, wm, wn, lane);
            } else if (g.transposed != 0) {
                float *ct = reinterpret_cast<float *>(g.C);
                const bool add = EPI == kEpiAccumF32 && g.accumulate != 0;
                if (edge) store_tile_transposed<true>(acc, ct, g.ldc, m0, n0, M, N, wm, wn, lane, add);
                else store_tile_transposed<false>(acc, ct, g.ldc, m0, n0, M, N, wm, wn, lane, add);
            } else if (edge) {
                store_tile<EPI, true>(acc, g.C, g.ldc, m0, n0, M, N, wm, wn, lane, g.accumulate != 0);
            } else if constexpr (EPI == kEpiAccumF32) {
                if (g.accumulate != 0) store_tile<EPI, false>(acc, g.C, g.ldc, m0, n0, M, N, wm, wn, lane, true);
                else store_tile_wide<EPI>(acc, g.C, g.ldc, m0, n0, wm, wn, lane, stage_tile);
            } else {
                store_tile_wide<EPI>(acc, g.C, g.ldc, m0, n0, wm, wn, lane, stage_tile);
            }
        }
        if constexpr (LSE) {
            const bool ragged = m0 + kGemmTile > M;
            const int mlim = (int)(M - m0) - wm * 128 - (lane >> 4) * 4;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (ragged) fold_column<true>(acc, b, mlim, run_m[b], run_s[b]);
                else fold_column<false>(acc, b, mlim, run_m[b], run_s[b]);
                __builtin_amdgcn_sched_barrier(0);
            }
            // end of this column group's sweep: merge the four lane groups, then the two row halves, and write the
            // workgroup's partial of its 256 columns (the reduction has LDS of its own: the ring keeps running)
            if (p_next >= p_end || (int)(p_next / rounds) != grp) {
                float2 *red = reinterpret_cast<float2 *>(lds + kDmaRingBytes);  // [2][256]
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    MaxSum mine = {run_m[b], run_s[b]};
#pragma unroll
                    for (int off = 16; off <= 32; off <<= 1) {
                        const MaxSum other = {__shfl_xor(mine.m, off, kWave), __shfl_xor(mine.s, off, kWave)};
                        mine = combine(mine, other);
                    }
                    if (lane < 16) red[wm * kGemmTile + wn * 64 + b * 16 + lane] = make_float2(mine.m, mine.s);
                    run_m[b] = kNegFloor;
                    run_s[b] = 0.0f;
                }
                // (the empty asm statements keep the compiler from moving LDS accesses across the bare barriers)
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(kNoVmWait, 0));
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (tid < kGemmTile) {
                    const float2 q0 = red[tid], q1 = red[kGemmTile + tid];
                    const MaxSum tot = combine(MaxSum{q0.x, q0.y}, MaxSum{q1.x, q1.y});
                    if (n0 + tid < N)
                        g.partial[(int64_t)(xcd * g.ml_count + ml) * g.partial_stride + n0 + tid] = make_float2(tot.m, tot.s);
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(kNoVmWait, 0));  // red is read before anyone writes it again
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
        }
        p_cur = p_next;
    }
    // drain: the reloads past the last stage must have landed before the workgroup ends
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
    __builtin_amdgcn_s_barrier();
}

// Sets every (max, sum) partial to the neutral element, so that slots no workgroup writes (an XCD that did not
// touch a column group) drop out of the merge.
__global__ void gemm_partials_init_kernel(float2 *partial, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) partial[i] = make_float2(kNegFloor, 0.0f);
}

// ---------------------------------------------------------------------------------------
// host side

// Shape of the persistent grid on the current device: one workgroup per compute unit, dealt round-robin to the
// XCDs by the dispatcher (eight XCDs on the full chip; a partition with fewer than 64 compute units is one XCD).
GemmGrid gemm_grid()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    GemmGrid gg;
    gg.nxcd = (cus >= 64 && cus % 8 == 0) ? 8 : 1;
    gg.ml_count = cus / gg.nxcd / kGemmColTiles;
    if (gg.ml_count < 1) gg.ml_count = 1;
    if (gg.nxcd * gg.ml_count > kGemmMaxPartialSlots) gg.ml_count = kGemmMaxPartialSlots / gg.nxcd;
    gg.blocks = gg.nxcd * gg.ml_count * kGemmColTiles;
    return gg;
}

size_t gemm_partial_slots() { const GemmGrid gg = gemm_grid(); return (size_t)gg.nxcd * gg.ml_count; }

template <int EPI>
static hipError_t launch_gemm_t(GemmArgs g, hipStream_t s)
{
    const GemmGrid gg = gemm_grid();
    g.nxcd = gg.nxcd;
    g.ml_count = gg.ml_count;
    const bool quad = g.K % (kDmaK * kDmaStages) == 0;
    auto *kernel = quad ? gemm_nt_kernel<EPI, true> : gemm_nt_kernel<EPI, false>;
    static LdsLimitState lds_limit[2];  // (one per variant of this epilogue)
    const hipError_t attr_err = ensure_lds_limit(reinterpret_cast<const void *>(kernel), kGemmLdsBytes, lds_limit[quad]);
    if (attr_err != hipSuccess) return attr_err;
    if (EPI == kEpiLse || EPI == kEpiLseStore) {
        const int64_t n = (int64_t)gg.nxcd * gg.ml_count * g.partial_stride;
        hipLaunchKernelGGL(gemm_partials_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, g.partial, n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3(gg.blocks), dim3(kGemmThreads), kGemmLdsBytes, s, g);
    return hipGetLastError();
}

hipError_t launch_gemm_nt(const GemmArgs &g, int epilogue, hipStream_t s)
{
    // what the kernel's 32-bit offsets and its stage arithmetic assume
    if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.K % 64 != 0 || g.lda % 8 != 0 || g.ldb % 8 != 0 || g.lda < g.K ||
        g.ldb < g.K || g.lda > (1 << 22) || g.ldb > (1 << 22))
        return hipErrorInvalidValue;
    if (g.dyn_dim != kDynNone && (!g.dyn.n || (g.dyn_dim == kDynK && g.K % 128 != 0))) return hipErrorInvalidValue;
    if ((g.a_panel && g.lda % 64 != 0) || (g.b_panel && g.ldb % 64 != 0)) return hipErrorInvalidValue;
    if (g.transposed != 0 && (g.M % 4 != 0 || g.dyn_dim == kDynM || epilogue == kEpiLse)) return hipErrorInvalidValue;
    if (epilogue != kEpiLse && (g.ldc % 8 != 0 || (reinterpret_cast<uintptr_t>(g.C) & 15) != 0)) return hipErrorInvalidValue;
    switch (epilogue) {
        case kEpiLse: return launch_gemm_t<kEpiLse>(g, s);
        case kEpiLseStore: return launch_gemm_t<kEpiLseStore>(g, s);
        case kEpiStoreBf16: return launch_gemm_t<kEpiStoreBf16>(g, s);
        case kEpiAccumF32: return launch_gemm_t<kEpiAccumF32>(g, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace a3po
