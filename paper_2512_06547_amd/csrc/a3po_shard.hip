// Vocabulary-sharded variant of the token log-prob and of the gradient to the logits: the columns of
// the logits are split over P shards (a tensor-parallel LM head), each shard reduces its columns to
// one 16-byte partial per token, the partials of all shards are merged into lse / log pi / entropy,
// and each shard then writes its own slice of the gradient from the merged values.  Between the two
// vocabulary-wide kernels sits whatever exchanges the partials (nothing, on one GPU).
//
// A shard row is read once per vocabulary-wide kernel with 16-byte non-temporal accesses (the forward
// streams with several vectors in flight per thread, the backward works in bursts); nothing is kept
// between the two except the merged per-token scalars, so a shard row crosses HBM three times (read,
// read, write).  The same three kernels also serve the unsharded loss when a row is too long to stay
// in registers (the whole vocabulary as one shard).
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

// launch shape of the streaming forward and of the element-wise backward (overridable at build time
// for tuning sweeps)
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
constexpr int64_t kShardWaveRowBytes = 65536;     // forward: rows up to this size always go one wavefront per row

// ---------------------------------------------------------------------------------------
// partial (max, sum exp, chosen logit if owned, sum exp * z) of one shard, one workgroup per row
template <typename DT>
__global__ __launch_bounds__(kShardThreads) void shard_partials_kernel(const void *z, int64_t T, int64_t Vs, int64_t ld,
                                                                      const int32_t *__restrict__ chosen, int64_t v0,
                                                                      a3po_shard_partial *__restrict__ out,
                                                                      const TokenRecord *__restrict__ records, int vec)
{
    constexpr int EPV = DT::kPerVec;
    __shared__ float red[3 * kShardWaves];
    const int tid = threadIdx.x;
    const int nfull = (int)(Vs / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;

    for (int64_t row = blockIdx.x; row < T; row += gridDim.x) {
        if (records && records[row].y < 0) continue;  // not counted: the row is not read (uniform over the workgroup)
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        const int64_t yl = (int64_t)chosen[row] - v0;  // asked for first: its latency hides behind the row's loads
        MaxSumU acc;
        seed(acc);
        if (vec) {
            // every pass issues up to kShardUnroll loads per thread before the first fold, the ragged last
            // pass included (a shard row is often little more than one pass long)
            for (int idx = tid; idx < nfull; idx += kShardUnroll * kShardThreads) {
                uint4 v[kShardUnroll];
#pragma unroll
                for (int u = 0; u < kShardUnroll; ++u)
                    if (idx + u * kShardThreads < nfull) v[u] = stream_load(in_row + (size_t)(idx + u * kShardThreads) * 16);
#pragma unroll
                for (int u = 0; u < kShardUnroll; ++u) {
                    if (idx + u * kShardThreads < nfull) {
                        float f[EPV];
                        unpack<DT>(v[u], f);
                        fold<EPV>(acc, f);
                    }
                }
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
        // the gather is issued before the reduction's barriers, not after them
        const float zy = (tid == 0 && yl >= 0 && yl < Vs) ? load_elem<DT>(in_row, yl) : 0.0f;
        const MaxSumU tot = block_allreduce<kShardWaves>(acc, red);
        if (tid == 0) {
            a3po_shard_partial p;
            p.max = tot.m;
            p.sum_exp = tot.s;
            p.chosen_logit = zy;
            p.sum_exp_z = tot.u;
            out[row] = p;
        }
    }
}

// The same, one wavefront per row: for narrow shards (a row is a few passes of one wavefront) there is no
// barrier and no LDS in the row's path, and the 32 wavefronts of a compute unit run independently.
// Vector path only (16-byte aligned base and stride).
template <typename DT>
__global__ __launch_bounds__(kShardThreads) void shard_partials_wave_kernel(const void *z, int64_t T, int64_t Vs,
                                                                           int64_t ld,
                                                                           const int32_t *__restrict__ chosen,
                                                                           int64_t v0,
                                                                           a3po_shard_partial *__restrict__ out,
                                                                           const TokenRecord *__restrict__ records)
{
    constexpr int EPV = DT::kPerVec;
    const int lane = threadIdx.x & (kWave - 1);
    const int nfull = (int)(Vs / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;
    const int64_t nwaves = (int64_t)gridDim.x * kShardWaves;
    for (int64_t row = (int64_t)blockIdx.x * kShardWaves + threadIdx.x / kWave; row < T; row += nwaves) {
        if (records && records[row].y < 0) continue;  // uniform over the wavefront
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        const int64_t yl = (int64_t)chosen[row] - v0;
        MaxSumU acc;
        seed(acc);
        for (int idx = lane; idx < nfull; idx += kShardUnroll * kWave) {
            uint4 v[kShardUnroll];
#pragma unroll
            for (int u = 0; u < kShardUnroll; ++u)
                if (idx + u * kWave < nfull) v[u] = stream_load(in_row + (size_t)(idx + u * kWave) * 16);
#pragma unroll
            for (int u = 0; u < kShardUnroll; ++u) {
                if (idx + u * kWave < nfull) {
                    float f[EPV];
                    unpack<DT>(v[u], f);
                    fold<EPV>(acc, f);
                }
            }
        }
        for (int64_t j = (int64_t)nfull * EPV + lane; j < Vs; j += kWave) {
            float f[1] = {load_elem<DT>(in_row, j)};
            fold<1>(acc, f);
        }
        const float zy = (lane == 0 && yl >= 0 && yl < Vs) ? load_elem<DT>(in_row, yl) : 0.0f;
        const MaxSumU tot = wave_reduce(acc);
        if (lane == 0) {
            a3po_shard_partial p;
            p.max = tot.m;
            p.sum_exp = tot.s;
            p.chosen_logit = zy;
            p.sum_exp_z = tot.u;
            out[row] = p;
        }
    }
}

// merge of the P partials of each token (ascending shard order, so the result does not depend on
// the launch shape)
__global__ void shard_combine_kernel(const a3po_shard_partial *__restrict__ parts, int32_t P, int64_t T,
                                     const int32_t *__restrict__ chosen, int64_t V, float *logp, float *lse_out,
                                     float *ent_out, const TokenRecord *__restrict__ records)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    if (records && records[t].y < 0) {  // not counted: no partial was written
        logp[t] = 0.0f;
        if (lse_out) lse_out[t] = 0.0f;
        if (ent_out) ent_out[t] = 0.0f;
        return;
    }
    MaxSumU tot;
    seed(tot);
    float zy = 0.0f;
    for (int32_t p = 0; p < P; ++p) {
        const a3po_shard_partial q = parts[(int64_t)p * T + t];
        tot = combine(tot, MaxSumU{q.max, q.sum_exp, q.sum_exp_z});
        zy += q.chosen_logit;  // exactly one shard owns the chosen column; the others hold 0
    }
    const float log_s = logf(tot.s);
    const float lse = tot.m + log_s;
    const int32_t y = chosen[t];
    const bool ok = y >= 0 && (int64_t)y < V;
    logp[t] = ok ? (zy - tot.m) - log_s : 0.0f;  // not zy - lse: lse carries the rounding of a large maximum
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
                        for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw((f[e] - lse) * kLog2e);
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
                    for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw((f[e] - lse) * kLog2e);
                    o = pack<DT>(f);
                }
                stream_store(out_row + (size_t)idx * 16, o);
            }
            for (int64_t j = (int64_t)nfull * EPV + tid; j < Vs; j += kShardThreads)
                store_elem<DT>(out_row, j, dead ? 0.0f : neg_g * exp2_hw((load_elem<DT>(in_row, j) - lse) * kLog2e));
        } else {
            for (int64_t j = tid; j < Vs; j += kShardThreads)
                store_elem<DT>(out_row, j, dead ? 0.0f : neg_g * exp2_hw((load_elem<DT>(in_row, j) - lse) * kLog2e));
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
// The same gradient slice in bursts.  A workgroup of 1024 threads takes an item of up to 7 x 1024
// sixteen-byte vectors (112 KiB) - several whole shard rows when they are short, one row, or one column chunk
// of a long row - loads all of it into registers, then computes and stores all of it: the
// read-a-burst / write-a-burst rhythm of the fused row kernel, which HBM rewards over fine-grained
// interleaving of loads and stores (about 5.9 against 5.0 TB/s on the same matrix).  Nothing here needs a whole
// row at once (the log-sum-exp is an input), so the burst length is free: 5 to 8 vectors per thread run 4-7 %
// faster than the 19 a row of the fused kernel takes (measured on a full-width matrix, on a 1/8 shard of its own
// and on eight column views), shorter ones are slower again.
// Vector path only (16-byte aligned bases and stride).  Per-row scalars of the item's rows are
// evaluated by the first threads and handed over through LDS (double-buffered by item parity, so one
// barrier per item suffices); the chosen column's +g is added in registers by the thread that holds
// that element.  Items come from the workspace's queue counter.
constexpr int kBurstThreads = 1024;  // one workgroup per compute unit: halves and quarters (more, smaller bursts) are 6-8 % slower
constexpr int kBurstVec = 7;         // vectors per thread and item

// hides a value's origin from the optimizer, so that index arithmetic is redone where it is needed
// instead of being kept in registers across the bursts (there are none to spare)
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

struct BurstShape {
    int nvec_row;    // 16-byte vectors per shard row (the last one may be partial)
    int align;       // 1: a row's slots start at the 128-byte line that holds its first vector (see below)
    int slots_row;   // slots per row: nvec_row, or with align nvec_row + 7 rounded up to a multiple of 8
    int rows;        // rows per item (1 when a row is cut into chunks)
    int chunks;      // column chunks per row
    int chunk_vec;   // slots per chunk (a multiple of 8 with align)
    uint32_t magic;  // floor(2^32 / slots_row) + 1: i / slots_row == umulhi(i, magic) for i, slots_row < 2^16
    int64_t items;
};
// Slots and alignment.  A thread's k-th vector is slot k * 1024 + tid of the item, so a wavefront's store covers 64
// consecutive slots.  A column slice of a wider matrix starts where its column offset puts it - for a 1/8 shard of
// 151,936 bf16 columns at a multiple of 32 bytes only - and stores that straddle 128-byte lines cost 7 % of the
// bandwidth.  With `align`, slot 0 of a row is the vector at the start of the line that holds the row's first
// vector: up to 7 leading slots (the row's phase, from the gradient's address) and the slots past the row's end are
// idle, and every wavefront's 64 slots cover whole lines.  Narrow rows, where idle slots would outnumber the gain,
// keep slot = vector.
constexpr int kBurstAlignMinVec = 128;

// SINGLE: an item is one row (or one column chunk of a row): no index divisions in the bursts.
template <typename DT, bool SINGLE>
__global__ __launch_bounds__(kBurstThreads) void shard_bwd_burst_kernel(
    const void *z, void *dz, int64_t T, int64_t Vs, int64_t ld, int64_t v0, const TokenRecord *__restrict__ records,
    const float *__restrict__ logp_theta, const float *__restrict__ lse_in, int32_t current_version, float clip_eps,
    int prox_mode, const WsHeader *__restrict__ hdr, unsigned int *queue, RowOutputs out, BurstShape sh)
{
    constexpr int EPV = DT::kPerVec;
    __shared__ float s_negg[2][kBurstThreads], s_lse[2][kBurstThreads];
    __shared__ int s_ycol[2][kBurstThreads];  // chosen column inside the shard, or -1
    __shared__ unsigned int s_next[2];
    const int tid = threadIdx.x;
    const size_t row_bytes = (size_t)ld * DT::kBytes;
    const float inv_n = hdr->inv_n;
    const int rem = (int)(Vs % EPV);  // elements of the partial last vector of a row (0 = none)
    // phase of row r, in vectors: ((address of the gradient's row r) / 16) mod 8 = (phase_base + r * phase_step) mod 8
    const int phase_base = sh.align ? (int)((reinterpret_cast<uintptr_t>(dz) >> 4) & 7) : 0;
    const int phase_step = sh.align ? (int)((row_bytes >> 4) & 7) : 0;
    int par = 0;

    int64_t item = blockIdx.x;
    while (item < sh.items) {
        const int64_t r0 = (item / sh.chunks) * sh.rows;
        const int chunk = (int)(item % sh.chunks);
        const int c0 = chunk * sh.chunk_vec;                          // first slot column of the item
        const int cw = min(sh.chunk_vec, sh.slots_row - c0);          // slot columns of the item
        const int nrows = (int)min((int64_t)sh.rows, T - r0);
        const int nvec = nrows * cw;
        const int phase0 = (phase_base + (int)(r0 & 7) * phase_step) & 7;
        // slot i of the item -> row r (relative) and vector column c of that row (outside [0, nvec_row): idle)
#define A3PO_BURST_SLOT(i, r, c)                                              \
    const int r = SINGLE ? 0 : (int)__umulhi((uint32_t)(i), sh.magic);          \
    const int c = c0 + ((i) - r * cw) - ((phase0 + r * phase_step) & 7)
        if (tid == 0) s_next[par] = atomicAdd(queue, 1u);
        if (tid < nrows) {
            const int64_t row = r0 + tid;
            const TokenRecord cur = records[row];
            float g = 0.0f, lse = 0.0f;
            if (cur.y >= 0) {
                lse = lse_in[row];
                const TokenTerms tt =
                    token_terms(logp_theta[row], cur.lb, cur.ver, current_version, cur.A, clip_eps, inv_n, prox_mode);
                g = tt.g;
                if (chunk == 0) {
                    if (out.prox) out.prox[row] = tt.lp;
                    out.obj[row] = tt.obj;
                    out.iw[row] = tt.iw;
                    out.flags[row] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) |
                                               (tt.negative_staleness ? kFlagNegStale : 0));
                }
            } else if (chunk == 0) {
                if (out.prox) out.prox[row] = 0.0f;
                out.obj[row] = 0.0f;
                out.iw[row] = 0.0f;
                out.flags[row] = 0;
            }
            const int64_t yl = (int64_t)cur.y - v0;
            s_negg[par][tid] = -g;
            s_lse[par][tid] = lse;
            s_ycol[par][tid] = (cur.y >= 0 && yl >= 0 && yl < Vs) ? (int)yl : -1;
        }
        __syncthreads();
        const int64_t next = (int64_t)gridDim.x + (int64_t)s_next[par];

        // ---- which of this thread's vectors belong to a row with a gradient (one bit each), so that the
        // loads below are issued back to back without waiting on LDS in between ----
        uint32_t live = 0;
#pragma unroll
        for (int k = 0; k < kBurstVec; ++k) {
            const int i = opaque(k * kBurstThreads + tid);
            A3PO_BURST_SLOT(i, r, c);
            if (i < nvec && (unsigned)c < (unsigned)sh.nvec_row && s_negg[par][r] != 0.0f) live |= 1u << k;
        }
        // ---- the read burst (row and column of a vector are recomputed rather than kept in registers) ----
        uint4 v[kBurstVec];
#pragma unroll
        for (int k = 0; k < kBurstVec; ++k) {
            if (live >> k & 1u) {
                const int i = opaque(k * kBurstThreads + tid);
                A3PO_BURST_SLOT(i, r, c);
                v[k] = stream_load(reinterpret_cast<const char *>(z) + (size_t)(r0 + r) * row_bytes + (size_t)c * 16);
            }
        }
        // the whole workgroup finishes reading before anyone writes: phases of 16 wavefronts, not of one
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();
        // ---- the write burst ----
#pragma unroll
        for (int k = 0; k < kBurstVec; ++k) {
            const int i = opaque(k * kBurstThreads + tid);
            if (i >= nvec) continue;
            A3PO_BURST_SLOT(i, r, c);
            if ((unsigned)c >= (unsigned)sh.nvec_row) continue;
            const float neg_g = s_negg[par][r];
            char *dst = reinterpret_cast<char *>(dz) + (size_t)(r0 + r) * row_bytes + (size_t)c * 16;
            float f[EPV];
            if (neg_g != 0.0f) {
                const float lse = s_lse[par][r];
                unpack<DT>(v[k], f);
                const int ye = s_ycol[par][r] - c * EPV;  // the chosen column's place in this vector
#pragma unroll
                for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw((f[e] - lse) * kLog2e);
                if ((unsigned)ye < (unsigned)EPV) {  // one vector per row: a real branch, not eight selects per vector
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        if (e == ye) f[e] -= neg_g;  // + g
                }
            } else {
#pragma unroll
                for (int e = 0; e < EPV; ++e) f[e] = 0.0f;
            }
            if (rem != 0 && c == sh.nvec_row - 1) {  // partial last vector: the columns beyond belong to a neighbour
                for (int e = 0; e < rem; ++e) store_elem<DT>(dst, e, f[e]);
            } else {
                stream_store(dst, pack<DT>(f));
            }
        }
#undef A3PO_BURST_SLOT
        par ^= 1;
        item = next;
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
                                 int64_t v0, a3po_shard_partial *out, const TokenRecord *records, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(z) && (ld * esz) % 16 == 0;
    const unsigned cap = shard_grid(T);
    // one wavefront per row for narrow rows, and for any rows when there are enough of them to give every
    // resident wavefront its own; one workgroup per row otherwise (few long rows)
    if (vec && (Vs * esz <= kShardWaveRowBytes || T >= (int64_t)cap * kShardWaves)) {
        const int64_t blocks = (T + kShardWaves - 1) / kShardWaves;
        const unsigned grid = (unsigned)(blocks < (int64_t)cap ? blocks : cap);
        if (dt == A3PO_F32)
            hipLaunchKernelGGL((shard_partials_wave_kernel<F32>), dim3(grid), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                               chosen, v0, out, records);
        else
            hipLaunchKernelGGL((shard_partials_wave_kernel<Bf16>), dim3(grid), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                               chosen, v0, out, records);
        return hipGetLastError();
    }
    if (dt == A3PO_F32)
        hipLaunchKernelGGL((shard_partials_kernel<F32>), dim3(shard_grid(T)), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                           chosen, v0, out, records, vec);
    else
        hipLaunchKernelGGL((shard_partials_kernel<Bf16>), dim3(shard_grid(T)), dim3(kShardThreads), 0, s, z, T, Vs, ld,
                           chosen, v0, out, records, vec);
    return hipGetLastError();
}

hipError_t launch_shard_combine(const a3po_shard_partial *parts, int32_t P, int64_t T, const int32_t *chosen, int64_t V,
                                float *logp, float *lse, float *ent, const TokenRecord *records, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    hipLaunchKernelGGL(shard_combine_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, parts, P, T, chosen, V,
                       logp, lse, ent, records);
    return hipGetLastError();
}

static BurstShape burst_shape(int64_t T, int64_t Vs, int64_t esz)
{
    const int64_t cap = (int64_t)kBurstVec * kBurstThreads;
    BurstShape sh;
    sh.nvec_row = (int)((Vs * esz + 15) / 16);
    sh.align = sh.nvec_row >= kBurstAlignMinVec;
    sh.slots_row = sh.align ? (sh.nvec_row + 7 + 7) / 8 * 8 : sh.nvec_row;
    if (sh.slots_row <= cap) {
        sh.rows = (int)(cap / sh.slots_row < kBurstThreads ? cap / sh.slots_row : kBurstThreads);
        sh.chunks = 1;
        sh.chunk_vec = sh.slots_row;
    } else {  // (only rows wide enough to be aligned get here)
        sh.rows = 1;
        const int chunks = (int)((sh.slots_row + cap - 1) / cap);
        sh.chunk_vec = ((sh.slots_row + chunks - 1) / chunks + 7) / 8 * 8;  // <= cap: cap is a multiple of 8
        sh.chunks = (sh.slots_row + sh.chunk_vec - 1) / sh.chunk_vec;
    }
    sh.magic = (uint32_t)((1ull << 32) / (uint64_t)sh.slots_row + 1);  // slots_row >= 2; used only when rows > 1 (then cw == slots_row)
    sh.items = ((T + sh.rows - 1) / sh.rows) * sh.chunks;
    return sh;
}

int64_t shard_bwd_queue_items(int dt, int64_t T, int64_t Vs)
{
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    if (T <= 0 || Vs * esz <= 16) return 0;
    return burst_shape(T, Vs, esz).items;
}

hipError_t launch_shard_bwd_rows(const LossArgs &a, int64_t v0, const float *logp_theta, const float *lse, hipStream_t s)
{
    if (a.T == 0) return hipSuccess;
    const int64_t esz = a.dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(a.z) && aligned16(a.dz) && (a.ld * esz) % 16 == 0;
    const RowOutputs out = {nullptr, a.prox_out, a.ws_obj, a.ws_iw, nullptr, a.ws_flags};
    const WsHeader *hdr = reinterpret_cast<const WsHeader *>(a.ws_header);
    // bursts for rows of at least two vectors (the reciprocal that stands in for the division by the row
    // length does not exist for 1); the queue counter in the workspace header was zeroed by the prep kernel
    if (vec && a.V * esz > 16) {
        const BurstShape sh = burst_shape(a.T, a.V, esz);
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        const unsigned grid = (unsigned)(sh.items < cus ? sh.items : cus);
#define A3PO_BURST_LAUNCH(DT, SINGLE) \
    hipLaunchKernelGGL((shard_bwd_burst_kernel<DT, SINGLE>), dim3(grid), dim3(kBurstThreads), 0, s, a.z, a.dz, a.T, a.V, \
                       a.ld, v0, a.ws_records, logp_theta, lse, a.current_version, a.clip_eps, a.prox_mode, hdr, \
                       row_queue_of(a.ws_header), out, sh)
        if (a.dt == A3PO_F32) {
            if (sh.rows == 1) A3PO_BURST_LAUNCH(F32, true);
            else A3PO_BURST_LAUNCH(F32, false);
        } else {
            if (sh.rows == 1) A3PO_BURST_LAUNCH(Bf16, true);
            else A3PO_BURST_LAUNCH(Bf16, false);
        }
#undef A3PO_BURST_LAUNCH
        return hipGetLastError();
    }
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
