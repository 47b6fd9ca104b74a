// Vocabulary-wide kernels for gfx950: the fused A-3PO loss forward+backward over logit
// rows, and the forward-only token log-prob kernel.
//
// Fused kernel layout.  A workgroup of 1024 threads (16 wavefronts of 64, four per SIMD)
// owns one row at a time and keeps the whole row in vector registers between the forward
// reduction and the gradient write, so each live row crosses HBM exactly twice: one
// coalesced 16-byte-per-lane read, one coalesced 16-byte-per-lane write.  A row of
// 151,936 bfloat16 is 297 KiB = 19 sixteen-byte vectors per thread (76 VGPRs); it does
// not fit the 160 KiB LDS but does fit the 512 KiB register file of a compute unit.
// All loads of a row are issued before the first is consumed; the online (max, sum)
// update of each vector then runs while later vectors are still in flight, and the
// gradient of each vector is stored while the next is being computed.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kMaxVec = 20;  // 16-byte vectors per thread the fused kernel can hold

// ---------------------------------------------------------------------------------------
// block-wide (max,sum) all-reduce through LDS, two barriers; for the multi-pass kernels
template <int WAVES>
__device__ __forceinline__ MaxSum block_allreduce(MaxSum v, float *sm, float *ss)
{
    v = wave_reduce(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    __syncthreads();  // previous readers of sm/ss are done
    if (lane == 0) {
        sm[wave] = v.m;
        ss[wave] = v.s;
    }
    __syncthreads();
    MaxSum t = {sm[0], ss[0]};
#pragma unroll
    for (int w = 1; w < WAVES; ++w) t = combine(t, MaxSum{sm[w], ss[w]});
    return t;
}

// ---------------------------------------------------------------------------------------
// Fused forward+backward, register-resident rows.
//
// NSWEEP is the exact number of 1024-lane sweeps of 16-byte vectors a row needs:
// (NSWEEP-1)*1024 < ceil(V / elements-per-vector) <= NSWEEP*1024.  Sweeps 0..NSWEEP-2 are
// full and carry no predicate at all; only the last sweep is predicated (and holds the
// ragged tail when V is not a multiple of the vector width).
// Requires: 16-byte aligned bases, (ld * element size) % 16 == 0, blockDim.x == 1024.
// Rows are claimed from a device-wide queue (one atomic add per row): workgroup b starts with
// row b and then takes whatever row is next, so masked rows (cheap) and slower compute units
// balance out by themselves.  The queue counter is zeroed by the prep kernel.
// Loads and stores of logit rows are non-temporal: every byte is touched exactly once.
constexpr uint32_t kSweepBytes = kRowThreads * 16;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 stream_load(const char *p)
{
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ void stream_store(char *p, const uint4 &v)
{
    const u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t *>(p));
}

struct RowOutputs {
    float *logp, *prox, *obj, *iw;
    uint8_t *flags;
};

template <typename DT, int NSWEEP>
__global__ __launch_bounds__(kRowThreads) void loss_rows_kernel(
    const void *z, void *dz, int64_t T, int64_t V, int64_t ld, const TokenRecord *__restrict__ records,
    int32_t current_version, float clip_eps, const WsHeader *__restrict__ hdr, unsigned int *row_queue,
    RowOutputs out)
{
    constexpr int EPV = DT::kPerVec;
    constexpr int LAST = NSWEEP - 1;
    __shared__ float red_m[2][kRowWaves];
    __shared__ float red_s[2][kRowWaves];
    __shared__ unsigned int next_row[2];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const uint32_t voff = (uint32_t)tid * 16u;
    const int nfull = (int)(V / EPV);  // complete vectors in a row
    const int rem = (int)(V % EPV);    // elements in the ragged tail vector (0 = none)
    // this thread's vector of the last sweep, relative to the row's end
    const int last_idx = LAST * kRowThreads + tid;
    const bool last_full = last_idx < nfull;               // a complete vector
    const bool last_tail = rem != 0 && last_idx == nfull;  // the ragged tail vector
    const bool last_any = last_full || last_tail;
    const float inv_n = hdr->inv_n;
    const size_t row_bytes = (size_t)ld * DT::kBytes;
    int parity = 0;

    // Per-token inputs are uniform over the workgroup and come from the packed records the
    // prep kernel wrote (one 16-byte scalar load per row, fetched as soon as the row is known).
    int64_t row = blockIdx.x;
    TokenRecord nxt = {-1, 0, 0.0f, 0.0f};
    if (row < T) nxt = records[row];

    while (row < T) {
        const TokenRecord cur = nxt;
        const int32_t y = cur.y;
        const bool live = y >= 0;  // the prep kernel stores y = -1 for masked or invalid tokens
        // thread 0 claims this workgroup's next row; the answer is shared at the row's barrier
        unsigned int claimed = 0;
        if (tid == 0) claimed = atomicAdd(row_queue, 1u);
        __builtin_amdgcn_sched_barrier(0);
        char *out_row = reinterpret_cast<char *>(dz) + (size_t)row * row_bytes;
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;

        uint4 v[NSWEEP];
        float g = 0.0f, lse = 0.0f, zy = 0.0f;
        uint32_t zy_bits = 0;
        int64_t next = T;
        if (live) {  // uniform over the workgroup
            // ---- issue every load of the row: the chosen logit, the partial sweep, the full sweeps ----
            // (scheduling barriers pin the issue order so that the forward pass below can
            // consume vectors in arrival order while later ones are still in flight)
            zy_bits = load_raw<DT>(in_row, y);
            __builtin_amdgcn_sched_barrier(0);
            v[LAST] = neg_inf_vec<DT>();
            if (last_any) v[LAST] = stream_load(in_row + (size_t)LAST * kSweepBytes + voff);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < LAST; ++k) {
                v[k] = stream_load(in_row + (size_t)k * kSweepBytes + voff);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- forward: online (max, sum) per thread, in the order the loads were issued ----
            MaxSum acc = {kNegFloor, 0.0f};
            {
                float f[EPV];
                unpack<DT>(v[LAST], f);
                if (last_tail) {
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        if (e >= rem) f[e] = -INFINITY;
                }
                fold<EPV>(acc, f);
            }
            if (tid == 0) next_row[parity] = claimed;  // the claim was issued before the row's loads
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < LAST; ++k) {
                float f[EPV];
                unpack<DT>(v[k], f);
                fold<EPV>(acc, f);
                __builtin_amdgcn_sched_barrier(0);
            }
            zy = raw_to_float<DT>(zy_bits);
            acc = wave_reduce(acc);
            if (lane == 0) {
                red_m[parity][wave] = acc.m;
                red_s[parity][wave] = acc.s;
            }
            __syncthreads();
            MaxSum tot = {red_m[parity][0], red_s[parity][0]};
#pragma unroll
            for (int w = 1; w < kRowWaves; ++w) tot = combine(tot, MaxSum{red_m[parity][w], red_s[parity][w]});
            const int64_t upcoming = (int64_t)gridDim.x + (int64_t)__builtin_amdgcn_readfirstlane(next_row[parity]);
            parity ^= 1;
            if (upcoming < T) nxt = records[upcoming];  // scalar load, lands during the backward pass

            lse = tot.m + logf(tot.s);
            const float lt = zy - lse;
            const TokenTerms tt = token_terms(lt, cur.lb, cur.ver, current_version, cur.A, clip_eps, inv_n);
            g = tt.g;
            if (tid == 0) {
                out.logp[row] = lt;
                if (out.prox) out.prox[row] = tt.lp;
                out.obj[row] = tt.obj;
                out.iw[row] = tt.iw;
                out.flags[row] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) |
                                           (tt.negative_staleness ? kFlagNegStale : 0));
            }
            next = upcoming;
        } else {
            if (tid == 0) {
                next_row[parity] = claimed;
                out.logp[row] = 0.0f;
                if (out.prox) out.prox[row] = 0.0f;
                out.obj[row] = 0.0f;
                out.iw[row] = 0.0f;
                out.flags[row] = 0;
            }
            __syncthreads();
            next = (int64_t)gridDim.x + (int64_t)__builtin_amdgcn_readfirstlane(next_row[parity]);
            parity ^= 1;
            if (next < T) nxt = records[next];
        }

        if (g == 0.0f) {
            // masked, invalid id, clipped, zero advantage or empty batch: the gradient row is zero
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int k = 0; k < LAST; ++k) stream_store(out_row + (size_t)k * kSweepBytes + voff, zero);
            if (last_full) {
                stream_store(out_row + (size_t)LAST * kSweepBytes + voff, zero);
            } else if (last_tail) {
                for (int e = 0; e < rem; ++e) store_elem<DT>(out_row, (int64_t)nfull * EPV + e, 0.0f);
            }
            row = next;
            continue;
        }

        // ---- backward: dz = g * (onehot(y) - softmax(z)), written over the same lanes ----
        const float neg_g = -g;
        const float nlse = -lse * kLog2e;
#pragma unroll
        for (int k = 0; k < LAST; ++k) {
            float f[EPV];
            unpack<DT>(v[k], f);
#pragma unroll
            for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw(fmaf(f[e], kLog2e, nlse));
            stream_store(out_row + (size_t)k * kSweepBytes + voff, pack<DT>(f));
        }
        if (last_any) {
            float f[EPV];
            unpack<DT>(v[LAST], f);
#pragma unroll
            for (int e = 0; e < EPV; ++e) f[e] = neg_g * exp2_hw(fmaf(f[e], kLog2e, nlse));
            if (last_full) {
                stream_store(out_row + (size_t)LAST * kSweepBytes + voff, pack<DT>(f));
            } else {
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    if (e < rem) store_elem<DT>(out_row, (int64_t)nfull * EPV + e, f[e]);
            }
        }
        // The chosen column gets +g.  The thread that stored the vector holding column y
        // rewrites that one element afterwards (same thread, same address: program order).
        if (tid == ((y / EPV) & (kRowThreads - 1)))
            store_elem<DT>(out_row, y, neg_g * exp2_hw(fmaf(zy, kLog2e, nlse)) + g);
        row = next;
    }
}

// ---------------------------------------------------------------------------------------
// Multi-pass fallback for rows the fused kernel cannot hold (unaligned stride, very large
// V): element-wise accesses, three reads of the row (max, sum, gradient).  Same results up
// to summation order.  Any blockDim.x that is a multiple of 64 up to 1024.
template <typename DT>
__global__ __launch_bounds__(kRowThreads) void loss_rows_generic_kernel(const LossArgs a)
{
    __shared__ float sm[kRowWaves], ss[kRowWaves];
    const int tid = threadIdx.x;
    const int64_t V = a.V;
    const float inv_n = reinterpret_cast<const WsHeader *>(a.ws_header)->inv_n;
    const size_t row_bytes = (size_t)a.ld * DT::kBytes;

    for (int64_t row = blockIdx.x; row < a.T; row += gridDim.x) {
        const TokenRecord cur = a.ws_records[row];
        const int32_t y = cur.y;
        const bool live = y >= 0;
        char *out_row = reinterpret_cast<char *>(a.dz) + (size_t)row * row_bytes;
        const char *in_row = reinterpret_cast<const char *>(a.z) + (size_t)row * row_bytes;
        float g = 0.0f, lse = 0.0f;
        if (live) {
            float m = kNegFloor;
            for (int64_t j = tid; j < V; j += blockDim.x) m = fmaxf(m, load_elem<DT>(in_row, j));
            MaxSum t = block_allreduce<kRowWaves>(MaxSum{m, 0.0f}, sm, ss);
            const float M = t.m;
            float s = 0.0f;
            const float nm = -M * kLog2e;
            for (int64_t j = tid; j < V; j += blockDim.x) s += exp2_hw(fmaf(load_elem<DT>(in_row, j), kLog2e, nm));
            t = block_allreduce<kRowWaves>(MaxSum{M, s}, sm, ss);
            lse = t.m + logf(t.s);
            const float lt = load_elem<DT>(in_row, y) - lse;
            const TokenTerms tt = token_terms(lt, cur.lb, cur.ver, a.current_version, cur.A, a.clip_eps, inv_n);
            g = tt.g;
            if (tid == 0) {
                a.logp_out[row] = lt;
                if (a.prox_out) a.prox_out[row] = tt.lp;
                a.ws_obj[row] = tt.obj;
                a.ws_iw[row] = tt.iw;
                a.ws_flags[row] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) |
                                            (tt.negative_staleness ? kFlagNegStale : 0));
            }
        } else if (tid == 0) {
            a.logp_out[row] = 0.0f;
            if (a.prox_out) a.prox_out[row] = 0.0f;
            a.ws_obj[row] = 0.0f;
            a.ws_iw[row] = 0.0f;
            a.ws_flags[row] = 0;
        }
        __syncthreads();  // every read of an aliased row is done before it is overwritten
        if (g == 0.0f) {
            for (int64_t j = tid; j < V; j += blockDim.x) store_elem<DT>(out_row, j, 0.0f);
        } else {
            const float nlse = -lse * kLog2e;
            for (int64_t j = tid; j < V; j += blockDim.x) {
                float d = -g * exp2_hw(fmaf(load_elem<DT>(in_row, j), kLog2e, nlse));
                if (j == (int64_t)y) d += g;
                store_elem<DT>(out_row, j, d);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Forward only: log-sum-exp and chosen-token gather, one 256-thread workgroup per row,
// rows dealt round-robin.  `vec` selects 16-byte loads (aligned rows) or element loads.
constexpr int kFwdThreads = 256;
constexpr int kFwdWaves = kFwdThreads / kWave;
constexpr int kFwdUnroll = 4;

template <typename DT>
__global__ __launch_bounds__(kFwdThreads) void logprob_rows_kernel(const void *z, int64_t T, int64_t V, int64_t ld,
                                                                    const int32_t *chosen, float *logp, float *lse_out,
                                                                    void *chosen_logit, int vec)
{
    constexpr int EPV = DT::kPerVec;
    __shared__ float sm[kFwdWaves], ss[kFwdWaves];
    const int tid = threadIdx.x;
    const int nfull = (int)(V / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;

    for (int64_t row = blockIdx.x; row < T; row += gridDim.x) {
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        MaxSum acc = {kNegFloor, 0.0f};
        if (vec) {
            const uint4 *src = reinterpret_cast<const uint4 *>(in_row);
            int idx = tid;
            for (; idx + (kFwdUnroll - 1) * kFwdThreads < nfull; idx += kFwdUnroll * kFwdThreads) {
                uint4 v[kFwdUnroll];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) v[u] = src[idx + u * kFwdThreads];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) {
                    float f[EPV];
                    unpack<DT>(v[u], f);
                    fold<EPV>(acc, f);
                }
            }
            for (; idx < nfull; idx += kFwdThreads) {
                float f[EPV];
                unpack<DT>(src[idx], f);
                fold<EPV>(acc, f);
            }
            for (int64_t j = (int64_t)nfull * EPV + tid; j < V; j += kFwdThreads) {
                float f[1] = {load_elem<DT>(in_row, j)};
                fold<1>(acc, f);
            }
        } else {
            for (int64_t j = tid; j < V; j += kFwdThreads) {
                float f[1] = {load_elem<DT>(in_row, j)};
                fold<1>(acc, f);
            }
        }
        const MaxSum tot = block_allreduce<kFwdWaves>(acc, sm, ss);
        if (tid == 0) {
            const float lse = tot.m + logf(tot.s);
            const int32_t y = chosen[row];
            const bool ok = y >= 0 && (int64_t)y < V;
            if (lse_out) lse_out[row] = lse;
            logp[row] = ok ? load_elem<DT>(in_row, y) - lse : 0.0f;
            if (chosen_logit) {
                if constexpr (DT::kBytes == 4) {
                    reinterpret_cast<uint32_t *>(chosen_logit)[row] =
                        ok ? reinterpret_cast<const uint32_t *>(in_row)[y] : 0u;
                } else {
                    reinterpret_cast<uint16_t *>(chosen_logit)[row] =
                        ok ? reinterpret_cast<const uint16_t *>(in_row)[y] : (uint16_t)0;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// host side

static int device_cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    return n;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool rows_fit_on_chip(int dt, int64_t V, int64_t ld, const void *z, const void *dz)
{
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    const int64_t epv = 16 / esz;
    const int64_t nvec = (V + epv - 1) / epv;
    return aligned16(z) && aligned16(dz) && (ld * esz) % 16 == 0 && nvec <= (int64_t)kMaxVec * kRowThreads;
}

template <typename DT>
static hipError_t launch_loss_rows_t(const LossArgs &a, hipStream_t s)
{
    const int64_t nvec = (a.V + DT::kPerVec - 1) / DT::kPerVec;
    const int cus = device_cu_count();
    const unsigned grid = (unsigned)(a.T < (int64_t)cus ? a.T : (int64_t)cus);
    if (!rows_fit_on_chip(a.dt, a.V, a.ld, a.z, a.dz)) {
        hipLaunchKernelGGL((loss_rows_generic_kernel<DT>), dim3(grid * 2 > a.T ? (unsigned)a.T : grid * 2),
                           dim3(kRowThreads), 0, s, a);
        return hipGetLastError();
    }
    const int sweeps = (int)((nvec + kRowThreads - 1) / kRowThreads);
    const RowOutputs out = {a.logp_out, a.prox_out, a.ws_obj, a.ws_iw, a.ws_flags};
    switch (sweeps) {
#define A3PO_SWEEP_CASE(N) \
    case N: \
        hipLaunchKernelGGL((loss_rows_kernel<DT, N>), dim3(grid), dim3(kRowThreads), 0, s, a.z, a.dz, a.T, a.V, a.ld, \
                           a.ws_records, a.current_version, a.clip_eps, \
                           reinterpret_cast<const WsHeader *>(a.ws_header), row_queue_of(a.ws_header), out); \
        break;
        A3PO_SWEEP_CASE(1) A3PO_SWEEP_CASE(2) A3PO_SWEEP_CASE(3) A3PO_SWEEP_CASE(4) A3PO_SWEEP_CASE(5)
        A3PO_SWEEP_CASE(6) A3PO_SWEEP_CASE(7) A3PO_SWEEP_CASE(8) A3PO_SWEEP_CASE(9) A3PO_SWEEP_CASE(10)
        A3PO_SWEEP_CASE(11) A3PO_SWEEP_CASE(12) A3PO_SWEEP_CASE(13) A3PO_SWEEP_CASE(14) A3PO_SWEEP_CASE(15)
        A3PO_SWEEP_CASE(16) A3PO_SWEEP_CASE(17) A3PO_SWEEP_CASE(18) A3PO_SWEEP_CASE(19) A3PO_SWEEP_CASE(20)
#undef A3PO_SWEEP_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_loss_rows(const LossArgs &a, hipStream_t s)
{
    if (a.T == 0) return hipSuccess;
    return a.dt == A3PO_F32 ? launch_loss_rows_t<F32>(a, s) : launch_loss_rows_t<Bf16>(a, s);
}

hipError_t launch_token_logprobs(const void *z, int dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                                 float *logp, float *lse, void *chosen_logit, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(z) && (ld * esz) % 16 == 0;
    const int64_t want = (int64_t)device_cu_count() * 8;
    const unsigned grid = (unsigned)(T < want ? T : want);
    if (dt == A3PO_F32)
        hipLaunchKernelGGL((logprob_rows_kernel<F32>), dim3(grid), dim3(kFwdThreads), 0, s, z, T, V, ld, chosen, logp,
                           lse, chosen_logit, vec);
    else
        hipLaunchKernelGGL((logprob_rows_kernel<Bf16>), dim3(grid), dim3(kFwdThreads), 0, s, z, T, V, ld, chosen, logp,
                           lse, chosen_logit, vec);
    return hipGetLastError();
}

}  // namespace a3po
