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

// One vector of the backward pass: f (logits) -> f (gradient entries without the chosen column's +g),
// and for ENT the running sum of p_j z_j (elements past the row's end hold -inf: p = 0).
// p_j = exp(z_j - lse) is evaluated as exp2((z_j - m) log2e - log2 s) with m the row's maximum and s its
// sum of exp(z - m): the difference is taken before the scaling, so the exponent's rounding error is
// relative to (z_j - m), not to the magnitude of the logits.
template <int EPV, bool ENT>
__device__ __forceinline__ void backward_vec(float *f, float neg_g, float row_max, float nls2, float &pz)
{
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        const float p = exp2_hw(fmaf(f[e] - row_max, kLog2e, nls2));
        if constexpr (ENT) pz = fmaf(p, finite_floor(f[e]), pz);
        f[e] = neg_g * p;
    }
}

// Overwrites elements rem.. of a packed vector with -inf (the ragged tail of a row).
template <typename DT>
__device__ __forceinline__ void mask_tail(uint4 &v, int rem)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    if constexpr (DT::kBytes == 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e >= rem) w[e] = 0xFF800000u;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e >= rem) w[e >> 1] = (e & 1) ? ((w[e >> 1] & 0x0000FFFFu) | 0xFF800000u) : ((w[e >> 1] & 0xFFFF0000u) | 0x0000FF80u);
    }
    v = make_uint4(w[0], w[1], w[2], w[3]);
}

// ENT adds the policy entropy of each counted row, H = lse - sum_j p_j z_j.  The sum rides on the
// backward pass, which evaluates every p_j anyway: one extra multiply-add per element, wave
// partials in LDS, and thread 0 finishes the row's entropy after the *next* row's barrier (by then
// every wave has left the backward pass), so no barrier is added.
// The extra live values do not fit beside 19 resident vectors in 128 registers, so for long rows the
// ENT variant parks the first STASH vectors it consumes in LDS between the forward and the backward
// pass and issues the last STASH loads of the row only then, into the registers just freed
// (a load pipeline of depth NSWEEP - STASH instead of NSWEEP).
// Rows of at most kTwoRowSweeps sweeps (64 KiB) run as two workgroups per compute unit (64 registers each): one
// such row is too short a burst to keep the memory system busy between a workgroup's barrier, queue claim and
// per-token arithmetic (+12 % at 32,000 bfloat16 columns, +26 % at 16,000; with longer rows two workgroups are slower).
constexpr int kTwoRowSweeps = 4;
template <typename DT, int NSWEEP, bool ENT>
__global__ __launch_bounds__(kRowThreads, NSWEEP <= kTwoRowSweeps ? 8 : 4) void loss_rows_kernel(
    const void *z, void *dz, int64_t T, int64_t V, int64_t ld, const TokenRecord *__restrict__ records,
    int32_t current_version, float clip_eps, int prox_mode, const WsHeader *__restrict__ hdr,
    unsigned int *row_queue, RowOutputs out)
{
    constexpr int EPV = DT::kPerVec;
    constexpr int LAST = NSWEEP - 1;
    constexpr int STASH = (ENT && NSWEEP >= 16) ? 2 : 0;  // consumed first: v[LAST], v[0]; loaded late: v[LAST-2], v[LAST-1]
    __shared__ float red_m[2][kRowWaves];
    __shared__ float red_s[2][kRowWaves];
    __shared__ float ent_part[2][kRowWaves];
    __shared__ unsigned int next_row[2];
    __shared__ uint4 stash[STASH ? STASH : 1][STASH ? kRowThreads : 1];

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
    // entropy of the previous counted row, finished after this row's barrier
    int64_t pend_row = -1;
    float pend_lse = 0.0f;
    int pend_par = 0;
    auto finish_pending_entropy = [&]() {
        if (pend_row >= 0 && tid == 0) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < kRowWaves; ++w) sum += ent_part[pend_par][w];
            out.ent[pend_row] = pend_lse - sum;
        }
        pend_row = -1;
    };

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
        const int row_par = parity;

        uint4 v[NSWEEP];
        float g = 0.0f, lse = 0.0f, zy = 0.0f, row_max = 0.0f, nls2 = 0.0f;
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
            for (int k = 0; k < LAST - STASH; ++k) {
                v[k] = stream_load(in_row + (size_t)k * kSweepBytes + voff);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- forward: online (max, sum) per thread, in the order the loads were issued ----
            MaxSum acc = {kNegFloor, 0.0f};
            {
                if (last_tail) mask_tail<DT>(v[LAST], rem);  // once; the backward pass sees the same -inf
                float f[EPV];
                unpack<DT>(v[LAST], f);
                fold<EPV>(acc, f);
                if constexpr (STASH > 0) {
                    stash[0][tid] = v[LAST];
                    v[LAST - STASH] = stream_load(in_row + (size_t)(LAST - STASH) * kSweepBytes + voff);
                }
            }
            if (tid == 0) next_row[parity] = claimed;  // the claim was issued before the row's loads
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < LAST; ++k) {
                float f[EPV];
                unpack<DT>(v[k], f);
                fold<EPV>(acc, f);
                if constexpr (STASH > 1) {
                    if (k + 1 < STASH) {
                        stash[k + 1][tid] = v[k];
                        v[LAST - STASH + k + 1] =
                            stream_load(in_row + (size_t)(LAST - STASH + k + 1) * kSweepBytes + voff);
                    }
                }
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
            if constexpr (ENT) finish_pending_entropy();

            row_max = tot.m;
            const float log_s = logf(tot.s);
            nls2 = -log_s * kLog2e;
            lse = tot.m + log_s;
            const float lt = (zy - tot.m) - log_s;  // not zy - lse: lse carries the rounding of a large maximum
            const TokenTerms tt =
                token_terms(lt, cur.lb, cur.ver, current_version, cur.A, clip_eps, inv_n, prox_mode);
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
                if constexpr (ENT) out.ent[row] = 0.0f;
                out.obj[row] = 0.0f;
                out.iw[row] = 0.0f;
                out.flags[row] = 0;
            }
            __syncthreads();
            next = (int64_t)gridDim.x + (int64_t)__builtin_amdgcn_readfirstlane(next_row[parity]);
            parity ^= 1;
            if (next < T) nxt = records[next];
            if constexpr (ENT) finish_pending_entropy();
        }

        const bool want_p = ENT ? live : g != 0.0f;  // the entropy needs every p_j of a counted row
        if (!want_p) {
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
        // (with ENT a counted row whose g is 0 comes through here too and stores exact zeros)
        // (+0 rather than -0 when there is no gradient: the row is then stored as +0 bit for bit, as the zero path does)
        const float neg_g = g != 0.0f ? -g : 0.0f;
        float pz = 0.0f;
#pragma unroll
        for (int k = (STASH > 1 ? STASH - 1 : 0); k < LAST; ++k) {
            float f[EPV];
            unpack<DT>(v[k], f);
            backward_vec<EPV, ENT>(f, neg_g, row_max, nls2, pz);
            stream_store(out_row + (size_t)k * kSweepBytes + voff, pack<DT>(f));
            if constexpr (ENT) __builtin_amdgcn_sched_barrier(0);  // one vector's temporaries at a time
        }
        if constexpr (STASH > 1) {  // the vectors parked in LDS come last, into registers that are free by now
#pragma unroll
            for (int k = 0; k < STASH - 1; ++k) {
                float f[EPV];
                unpack<DT>(stash[k + 1][tid], f);
                backward_vec<EPV, ENT>(f, neg_g, row_max, nls2, pz);
                stream_store(out_row + (size_t)k * kSweepBytes + voff, pack<DT>(f));
            }
        }
        if (last_any) {
            float f[EPV];
            if constexpr (STASH > 0) unpack<DT>(stash[0][tid], f);
            else unpack<DT>(v[LAST], f);
            backward_vec<EPV, ENT>(f, neg_g, row_max, nls2, pz);
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
        if (g != 0.0f && tid == ((y / EPV) & (kRowThreads - 1)))
            store_elem<DT>(out_row, y, neg_g * exp2_hw(fmaf(zy - row_max, kLog2e, nls2)) + g);
        if constexpr (ENT) {
#pragma unroll
            for (int off = kWave / 2; off > 0; off >>= 1) pz += __shfl_xor(pz, off, kWave);
            if (lane == 0) ent_part[row_par][wave] = pz;
            pend_row = row;
            pend_lse = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(lse)));
            pend_par = row_par;
        }
        row = next;
    }
    if constexpr (ENT) {
        __syncthreads();
        finish_pending_entropy();
    }
}

// ---------------------------------------------------------------------------------------
// Fused forward+backward for rows that do not fit the registers (more than kMaxVec sweeps: fp32 logits at the
// full vocabulary, bfloat16 beyond 163,840 columns).  Same workgroup per row, same queue, same arithmetic; the
// row is cut into three parts by sweep index:
//   sweeps 0 .. kLongReg-1            in vector registers, as in the kernel above;
//   the next up to kLongLds sweeps    in LDS, brought there by direct global -> LDS loads (no registers, no LDS
//                                     write instructions; lane l of a wavefront lands at base + 16 l, so a thread
//                                     reads back exactly the 16 bytes its own load wrote and no barrier is needed);
//   the rest ("tail")                 streamed: read once for the forward reduction, last of all, and read again
//                                     at the end of the backward pass, latest sweeps first.
// Registers plus LDS hold 28 sweeps = 448 KiB, three quarters of an fp32 row of 151,936 (594 KiB): at most 2.25
// crossings of HBM per row instead of the 3 of separate forward and backward passes.  The first read of the tail
// is an ordinary load and most of the second reading is then served by the caches (with a non-temporal first read
// the kernel is 10 % slower); everything else is non-temporal.
constexpr int kLongReg = 19;     // sweeps in registers
constexpr int kLongRegEnt = 15;  // the same with the entropy, whose running sum and temporaries need the room
constexpr int kLongLds = 9;
constexpr int kLongTailUnroll = 4;  // tail vectors in flight per thread
constexpr int kLongStashBytes = kLongLds * (int)kSweepBytes;
constexpr int kLongLdsBytes = kLongStashBytes + (6 * kRowWaves + 2) * (int)sizeof(float);

typedef __attribute__((address_space(3))) void *rows_lds_ptr_t;

__device__ __forceinline__ uint4 cached_load(const char *p) { return *reinterpret_cast<const uint4 *>(p); }

template <typename DT, bool ENT>
__global__ __launch_bounds__(kRowThreads) void loss_rows_long_kernel(
    const void *z, void *dz, int64_t T, int64_t V, int64_t ld, const TokenRecord *__restrict__ records,
    int32_t current_version, float clip_eps, int prox_mode, const WsHeader *__restrict__ hdr,
    unsigned int *row_queue, RowOutputs out)
{
    constexpr int EPV = DT::kPerVec;
    constexpr int NREG = ENT ? kLongRegEnt : kLongReg;
    extern __shared__ __align__(16) char smem[];
    float *red_m = reinterpret_cast<float *>(smem + kLongStashBytes);  // [2][kRowWaves]
    float *red_s = red_m + 2 * kRowWaves;
    float *ent_part = red_s + 2 * kRowWaves;                           // [2][kRowWaves]
    unsigned int *next_row = reinterpret_cast<unsigned int *>(ent_part + 2 * kRowWaves);  // [2]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t voff = (uint32_t)tid * 16u;
    const int nfull = (int)(V / EPV);
    const int rem = (int)(V % EPV);
    const int nvec = nfull + (rem != 0);
    const int nsweep = (nvec + kRowThreads - 1) / kRowThreads;                    // > kMaxVec
    const int lds_sweeps = min(kLongLds, nsweep - NREG);                      // >= 2
    const int tail0 = NREG + lds_sweeps;                                      // first streamed sweep
    const int tail_batches = (nsweep - tail0 + kLongTailUnroll - 1) / kLongTailUnroll;
    const float inv_n = hdr->inv_n;
    const size_t row_bytes = (size_t)ld * DT::kBytes;
    char *my_stash = smem + voff;  // + j * kSweepBytes: this thread's vector of LDS sweep j
    int parity = 0;
    // entropy of the previous counted row, finished after this row's barrier (as in the kernel above)
    int64_t pend_row = -1;
    float pend_lse = 0.0f;
    int pend_par = 0;
    auto finish_pending_entropy = [&]() {
        if (pend_row >= 0 && tid == 0) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < kRowWaves; ++w) sum += ent_part[pend_par * kRowWaves + w];
            out.ent[pend_row] = pend_lse - sum;
        }
        pend_row = -1;
    };

    int64_t row = blockIdx.x;
    TokenRecord nxt = {-1, 0, 0.0f, 0.0f};
    if (row < T) nxt = records[row];

    while (row < T) {
        const TokenRecord cur = nxt;
        const int32_t y = cur.y;
        const bool live = y >= 0;
        unsigned int claimed = 0;
        if (tid == 0) claimed = atomicAdd(row_queue, 1u);
        __builtin_amdgcn_sched_barrier(0);
        char *out_row = reinterpret_cast<char *>(dz) + (size_t)row * row_bytes;
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        const int row_par = parity;

        uint4 v[NREG];
        float g = 0.0f, lse = 0.0f, zy = 0.0f, row_max = 0.0f, nls2 = 0.0f;
        int64_t next = T;
        if (live) {
            // a copy of the thread index the compiler cannot see through: the addresses of the direct loads are
            // then computed where they are used (two instructions each) instead of being kept, and spilled,
            // across the whole row loop
            int tid_r = tid;
            asm volatile("" : "+v"(tid_r));
            const uint32_t zy_bits = load_raw<DT>(in_row, y);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < NREG; ++k) {
                v[k] = stream_load(in_row + (size_t)k * kSweepBytes + voff);
                __builtin_amdgcn_sched_barrier(0);
            }
            // LDS sweeps; a lane past the row's end fetches the row's last vector instead (its data is never used)
#pragma unroll
            for (int j = 0; j < kLongLds; ++j) {
                if (j < lds_sweeps) {
                    const uint32_t idx = (uint32_t)min((NREG + j) * kRowThreads + tid_r, nvec - 1);
                    __builtin_amdgcn_global_load_lds(reinterpret_cast<const u32x4_t *>(in_row + (size_t)(idx * 16u)),
                                                     (rows_lds_ptr_t)(smem + j * (int)kSweepBytes + wave_s * 1024), 16, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }

            MaxSum acc = {kNegFloor, 0.0f};
            if (tid == 0) next_row[parity] = claimed;
#pragma unroll
            for (int k = 0; k < NREG; ++k) {
                float f[EPV];
                unpack<DT>(v[k], f);
                fold<EPV>(acc, f);
                __builtin_amdgcn_sched_barrier(0);
            }
            // the direct loads are invisible to the compiler's dependency tracking: wait for them by hand
            __builtin_amdgcn_s_waitcnt(0x0070 | (15 << 8));  // vmcnt(0), LDS count untouched
            __builtin_amdgcn_sched_barrier(0);
            for (int j = 0; j < lds_sweeps; ++j) {
                const int idx = (NREG + j) * kRowThreads + tid;
                uint4 t = *reinterpret_cast<const uint4 *>(my_stash + j * (int)kSweepBytes);
                if (idx >= nvec) {
                    t = neg_inf_vec<DT>();
                } else if (rem != 0 && idx == nfull) {  // the ragged tail vector: -inf past the row's end, once
                    mask_tail<DT>(t, rem);
                    *reinterpret_cast<uint4 *>(my_stash + j * (int)kSweepBytes) = t;
                }
                float f[EPV];
                unpack<DT>(t, f);
                fold<EPV>(acc, f);
            }
            // tail, first reading
            for (int b = 0; b < tail_batches; ++b) {
                uint4 t[kLongTailUnroll];
#pragma unroll
                for (int u = 0; u < kLongTailUnroll; ++u) {
                    const int idx = (tail0 + b * kLongTailUnroll + u) * kRowThreads + tid;
                    t[u] = neg_inf_vec<DT>();
                    if (idx < nvec) t[u] = cached_load(in_row + (size_t)idx * 16);
                }
#pragma unroll
                for (int u = 0; u < kLongTailUnroll; ++u) {
                    const int idx = (tail0 + b * kLongTailUnroll + u) * kRowThreads + tid;
                    if (rem != 0 && idx == nfull) mask_tail<DT>(t[u], rem);
                    float f[EPV];
                    unpack<DT>(t[u], f);
                    fold<EPV>(acc, f);
                }
            }
            zy = raw_to_float<DT>(zy_bits);
            acc = wave_reduce(acc);
            if (lane == 0) {
                red_m[parity * kRowWaves + wave] = acc.m;
                red_s[parity * kRowWaves + wave] = acc.s;
            }
            __syncthreads();
            MaxSum tot = {red_m[parity * kRowWaves], red_s[parity * kRowWaves]};
#pragma unroll
            for (int w = 1; w < kRowWaves; ++w)
                tot = combine(tot, MaxSum{red_m[parity * kRowWaves + w], red_s[parity * kRowWaves + w]});
            const int64_t upcoming = (int64_t)gridDim.x + (int64_t)__builtin_amdgcn_readfirstlane(next_row[parity]);
            parity ^= 1;
            if (upcoming < T) nxt = records[upcoming];
            if constexpr (ENT) finish_pending_entropy();

            row_max = tot.m;
            const float log_s = logf(tot.s);
            nls2 = -log_s * kLog2e;
            lse = tot.m + log_s;
            const float lt = (zy - tot.m) - log_s;
            const TokenTerms tt =
                token_terms(lt, cur.lb, cur.ver, current_version, cur.A, clip_eps, inv_n, prox_mode);
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
                if constexpr (ENT) out.ent[row] = 0.0f;
                out.obj[row] = 0.0f;
                out.iw[row] = 0.0f;
                out.flags[row] = 0;
            }
            __syncthreads();
            next = (int64_t)gridDim.x + (int64_t)__builtin_amdgcn_readfirstlane(next_row[parity]);
            parity ^= 1;
            if (next < T) nxt = records[next];
            if constexpr (ENT) finish_pending_entropy();
        }

        const bool want_p = ENT ? live : g != 0.0f;  // the entropy needs every p_j of a counted row
        if (!want_p) {
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            for (int k = 0; k < nsweep; ++k) {
                const int idx = k * kRowThreads + tid;
                if (idx < nfull) {
                    stream_store(out_row + (size_t)idx * 16, zero);
                } else if (idx == nfull) {
                    for (int e = 0; e < rem; ++e) store_elem<DT>(out_row, (int64_t)nfull * EPV + e, 0.0f);
                }
            }
            row = next;
            continue;
        }

        const float neg_g = g != 0.0f ? -g : 0.0f;  // +0 rows when there is no gradient, as the zero path stores
        float pz = 0.0f;
        auto emit = [&](uint4 t, int idx) {  // gradient of one vector; idx < nvec
            float f[EPV];
            unpack<DT>(t, f);
            backward_vec<EPV, ENT>(f, neg_g, row_max, nls2, pz);
            if (idx < nfull) {
                stream_store(out_row + (size_t)idx * 16, pack<DT>(f));
            } else {
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    if (e < rem) store_elem<DT>(out_row, (int64_t)nfull * EPV + e, f[e]);
            }
        };
#pragma unroll
        for (int k = 0; k < NREG; ++k) {
            float f[EPV];
            unpack<DT>(v[k], f);
            backward_vec<EPV, ENT>(f, neg_g, row_max, nls2, pz);
            stream_store(out_row + (size_t)k * kSweepBytes + voff, pack<DT>(f));
            if constexpr (ENT) __builtin_amdgcn_sched_barrier(0);  // one vector's temporaries at a time
        }
        for (int j = 0; j < lds_sweeps; ++j) {
            const int idx = (NREG + j) * kRowThreads + tid;
            if (idx < nvec) emit(*reinterpret_cast<const uint4 *>(my_stash + j * (int)kSweepBytes), idx);
        }
        // tail, second reading: latest sweeps first
        for (int b = tail_batches - 1; b >= 0; --b) {
            uint4 t[kLongTailUnroll];
#pragma unroll
            for (int u = 0; u < kLongTailUnroll; ++u) {
                const int idx = (tail0 + b * kLongTailUnroll + u) * kRowThreads + tid;
                t[u] = neg_inf_vec<DT>();
                if (idx < nvec) t[u] = stream_load(in_row + (size_t)idx * 16);
            }
#pragma unroll
            for (int u = 0; u < kLongTailUnroll; ++u) {
                const int idx = (tail0 + b * kLongTailUnroll + u) * kRowThreads + tid;
                if (idx < nvec) {
                    if (rem != 0 && idx == nfull) mask_tail<DT>(t[u], rem);
                    emit(t[u], idx);
                }
            }
        }
        // the chosen column gets +g from the thread that stored its vector (same thread, same address: program order)
        if (g != 0.0f && tid == ((y / EPV) & (kRowThreads - 1)))
            store_elem<DT>(out_row, y, neg_g * exp2_hw(fmaf(zy - row_max, kLog2e, nls2)) + g);
        if constexpr (ENT) {
#pragma unroll
            for (int off = kWave / 2; off > 0; off >>= 1) pz += __shfl_xor(pz, off, kWave);
            if (lane == 0) ent_part[row_par * kRowWaves + wave] = pz;
            pend_row = row;
            pend_lse = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(lse)));
            pend_par = row_par;
        }
        row = next;
    }
    if constexpr (ENT) {
        __syncthreads();
        finish_pending_entropy();
    }
}

// ---------------------------------------------------------------------------------------
// Multi-pass fallback for rows the fused kernel cannot hold (unaligned stride, very large
// V): element-wise accesses, three reads of the row (max, sum, gradient).  Same results up
// to summation order.  Any blockDim.x that is a multiple of 64 up to 1024.
template <typename DT>
__global__ __launch_bounds__(kRowThreads) void loss_rows_generic_kernel(const LossArgs a)
{
    __shared__ float red[3 * kRowWaves];
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
        float g = 0.0f, lse = 0.0f, row_max = 0.0f, nls2 = 0.0f;
        if (live) {
            float m = kNegFloor;
            for (int64_t j = tid; j < V; j += blockDim.x) m = fmaxf(m, load_elem<DT>(in_row, j));
            const float M = block_allreduce<kRowWaves>(MaxSum{m, 0.0f}, red).m;
            float s = 0.0f, u = 0.0f;
            for (int64_t j = tid; j < V; j += blockDim.x) {
                const float zj = load_elem<DT>(in_row, j);
                const float ex = exp2_hw((zj - M) * kLog2e);
                s += ex;
                u = fmaf(ex, finite_floor(zj), u);
            }
            const MaxSumU t = block_allreduce<kRowWaves>(MaxSumU{M, s, u}, red);
            row_max = t.m;
            const float log_s = logf(t.s);
            nls2 = -log_s * kLog2e;
            lse = t.m + log_s;
            const float lt = (load_elem<DT>(in_row, y) - t.m) - log_s;
            const TokenTerms tt =
                token_terms(lt, cur.lb, cur.ver, a.current_version, cur.A, a.clip_eps, inv_n, a.prox_mode);
            g = tt.g;
            if (tid == 0) {
                a.logp_out[row] = lt;
                if (a.prox_out) a.prox_out[row] = tt.lp;
                if (a.ent_out) a.ent_out[row] = entropy_of(t, lse);
                a.ws_obj[row] = tt.obj;
                a.ws_iw[row] = tt.iw;
                a.ws_flags[row] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) |
                                            (tt.negative_staleness ? kFlagNegStale : 0));
            }
        } else if (tid == 0) {
            a.logp_out[row] = 0.0f;
            if (a.prox_out) a.prox_out[row] = 0.0f;
            if (a.ent_out) a.ent_out[row] = 0.0f;
            a.ws_obj[row] = 0.0f;
            a.ws_iw[row] = 0.0f;
            a.ws_flags[row] = 0;
        }
        __syncthreads();  // every read of an aliased row is done before it is overwritten
        if (g == 0.0f) {
            for (int64_t j = tid; j < V; j += blockDim.x) store_elem<DT>(out_row, j, 0.0f);
        } else {
            for (int64_t j = tid; j < V; j += blockDim.x) {
                float d = -g * exp2_hw(fmaf(load_elem<DT>(in_row, j) - row_max, kLog2e, nls2));
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
constexpr int kFwdUnroll = 8;  // 16-byte vectors in flight per thread

template <typename DT, bool ENT>
__global__ __launch_bounds__(kFwdThreads) void logprob_rows_kernel(const void *z, int64_t T, int64_t V, int64_t ld,
                                                                    const int32_t *chosen, float *logp, float *lse_out,
                                                                    void *chosen_logit, float *ent_out, int vec)
{
    constexpr int EPV = DT::kPerVec;
    using Acc = typename RowAcc<ENT>::type;
    __shared__ float red[3 * kFwdWaves];
    const int tid = threadIdx.x;
    const int nfull = (int)(V / EPV);
    const size_t row_bytes = (size_t)ld * DT::kBytes;

    for (int64_t row = blockIdx.x; row < T; row += gridDim.x) {
        const char *in_row = reinterpret_cast<const char *>(z) + (size_t)row * row_bytes;
        Acc acc;
        seed(acc);
        if (vec) {
            int idx = tid;
            for (; idx + (kFwdUnroll - 1) * kFwdThreads < nfull; idx += kFwdUnroll * kFwdThreads) {
                uint4 v[kFwdUnroll];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) v[u] = stream_load(in_row + (size_t)(idx + u * kFwdThreads) * 16);
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) {
                    float f[EPV];
                    unpack<DT>(v[u], f);
                    fold<EPV>(acc, f);
                }
            }
            for (; idx < nfull; idx += kFwdThreads) {
                float f[EPV];
                unpack<DT>(stream_load(in_row + (size_t)idx * 16), f);
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
        const Acc tot = block_allreduce<kFwdWaves>(acc, red);
        if (tid == 0) {
            const float log_s = logf(tot.s);
            const float lse = tot.m + log_s;
            const int32_t y = chosen[row];
            const bool ok = y >= 0 && (int64_t)y < V;
            if (lse_out) lse_out[row] = lse;
            if constexpr (ENT) ent_out[row] = entropy_of(tot, lse);
            logp[row] = ok ? (load_elem<DT>(in_row, y) - tot.m) - log_s : 0.0f;
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
        if (aligned16(a.z) && aligned16(a.dz) && (a.ld * DT::kBytes) % 16 == 0) {
            // aligned but too long for the registers: registers + LDS + a streamed tail
            const RowOutputs lout = {a.logp_out, a.prox_out, a.ws_obj, a.ws_iw, a.ent_out, a.ws_flags};
            const WsHeader *lhdr = reinterpret_cast<const WsHeader *>(a.ws_header);
            static LdsLimitState lds_limit[2];
            const void *kernel = a.ent_out ? reinterpret_cast<const void *>(&loss_rows_long_kernel<DT, true>)
                                           : reinterpret_cast<const void *>(&loss_rows_long_kernel<DT, false>);
            const hipError_t attr_err = ensure_lds_limit(kernel, kLongLdsBytes, lds_limit[a.ent_out ? 1 : 0]);
            if (attr_err != hipSuccess) return attr_err;
            if (a.ent_out)
                hipLaunchKernelGGL((loss_rows_long_kernel<DT, true>), dim3(grid), dim3(kRowThreads), kLongLdsBytes, s,
                                   a.z, a.dz, a.T, a.V, a.ld, a.ws_records, a.current_version, a.clip_eps, a.prox_mode,
                                   lhdr, row_queue_of(a.ws_header), lout);
            else
                hipLaunchKernelGGL((loss_rows_long_kernel<DT, false>), dim3(grid), dim3(kRowThreads), kLongLdsBytes, s,
                                   a.z, a.dz, a.T, a.V, a.ld, a.ws_records, a.current_version, a.clip_eps, a.prox_mode,
                                   lhdr, row_queue_of(a.ws_header), lout);
            return hipGetLastError();
        }
        hipLaunchKernelGGL((loss_rows_generic_kernel<DT>), dim3(grid * 2 > a.T ? (unsigned)a.T : grid * 2),
                           dim3(kRowThreads), 0, s, a);
        return hipGetLastError();
    }
    const int sweeps = (int)((nvec + kRowThreads - 1) / kRowThreads);
    const int64_t resident = (int64_t)cus * (sweeps <= kTwoRowSweeps ? 2 : 1);
    const unsigned row_grid = (unsigned)(a.T < resident ? a.T : resident);
    const RowOutputs out = {a.logp_out, a.prox_out, a.ws_obj, a.ws_iw, a.ent_out, a.ws_flags};
    const WsHeader *hdr = reinterpret_cast<const WsHeader *>(a.ws_header);
    unsigned int *queue = row_queue_of(a.ws_header);
    switch (sweeps) {
#define A3PO_SWEEP_CASE(N) \
    case N: \
        if (a.ent_out) \
            hipLaunchKernelGGL((loss_rows_kernel<DT, N, true>), dim3(row_grid), dim3(kRowThreads), 0, s, a.z, a.dz, a.T, \
                               a.V, a.ld, a.ws_records, a.current_version, a.clip_eps, a.prox_mode, hdr, queue, out); \
        else \
            hipLaunchKernelGGL((loss_rows_kernel<DT, N, false>), dim3(row_grid), dim3(kRowThreads), 0, s, a.z, a.dz, a.T, \
                               a.V, a.ld, a.ws_records, a.current_version, a.clip_eps, a.prox_mode, hdr, queue, out); \
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

template <typename DT>
static void launch_logprob_rows_t(unsigned grid, hipStream_t s, const void *z, int64_t T, int64_t V, int64_t ld,
                                  const int32_t *chosen, float *logp, float *lse, void *chosen_logit, float *ent,
                                  int vec)
{
    if (ent)
        hipLaunchKernelGGL((logprob_rows_kernel<DT, true>), dim3(grid), dim3(kFwdThreads), 0, s, z, T, V, ld, chosen,
                           logp, lse, chosen_logit, ent, vec);
    else
        hipLaunchKernelGGL((logprob_rows_kernel<DT, false>), dim3(grid), dim3(kFwdThreads), 0, s, z, T, V, ld, chosen,
                           logp, lse, chosen_logit, ent, vec);
}

hipError_t launch_token_logprobs(const void *z, int dt, int64_t T, int64_t V, int64_t ld, const int32_t *chosen,
                                 float *logp, float *lse, void *chosen_logit, float *ent, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const int64_t esz = dt == A3PO_F32 ? 4 : 2;
    const int vec = aligned16(z) && (ld * esz) % 16 == 0;
    const int64_t want = (int64_t)device_cu_count() * 8;
    const unsigned grid = (unsigned)(T < want ? T : want);
    if (dt == A3PO_F32) launch_logprob_rows_t<F32>(grid, s, z, T, V, ld, chosen, logp, lse, chosen_logit, ent, vec);
    else launch_logprob_rows_t<Bf16>(grid, s, z, T, V, ld, chosen, logp, lse, chosen_logit, ent, vec);
    return hipGetLastError();
}

}  // namespace a3po
