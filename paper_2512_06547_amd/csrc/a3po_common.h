// Device-side helpers shared by the gfx950 kernels: element packing, wave/block
// reductions for 64-wide wavefronts, and the per-token A-3PO arithmetic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "a3po.h"

namespace a3po {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegFloor = -1.0e30f;  // running-max seed; logits are assumed above this
constexpr int kWave = 64;

struct F32 {
    using scalar = float;
    static constexpr int kBytes = 4;
    static constexpr int kPerVec = 4;  // elements per 16-byte vector
};
struct Bf16 {
    using scalar = uint16_t;
    static constexpr int kBytes = 2;
    static constexpr int kPerVec = 8;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// two floats -> packed bfloat16 pair, round to nearest even (lo in bits 0..15)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_t f = {lo, hi};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <typename DT>
__device__ __forceinline__ uint4 neg_inf_vec()
{
    if constexpr (DT::kBytes == 4) return make_uint4(0xFF800000u, 0xFF800000u, 0xFF800000u, 0xFF800000u);
    else return make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u);
}

// widen one 16-byte vector to DT::kPerVec floats (exact)
template <typename DT>
__device__ __forceinline__ void unpack(const uint4 &v, float *f)
{
    if constexpr (DT::kBytes == 4) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    } else {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
}

template <typename DT>
__device__ __forceinline__ uint4 pack(const float *f)
{
    if constexpr (DT::kBytes == 4) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    } else {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                          pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
}

// one element (index e) of a row, widened exactly
template <typename DT>
__device__ __forceinline__ float load_elem(const void *row, int64_t e)
{
    if constexpr (DT::kBytes == 4) return reinterpret_cast<const float *>(row)[e];
    else return bf16_bits_to_float(reinterpret_cast<const uint16_t *>(row)[e]);
}

// stored bits of one element, zero-extended; raw_to_float widens them exactly
template <typename DT>
__device__ __forceinline__ uint32_t load_raw(const void *row, int64_t e)
{
    if constexpr (DT::kBytes == 4) return reinterpret_cast<const uint32_t *>(row)[e];
    else return reinterpret_cast<const uint16_t *>(row)[e];
}

template <typename DT>
__device__ __forceinline__ float raw_to_float(uint32_t bits)
{
    if constexpr (DT::kBytes == 4) return __uint_as_float(bits);
    else return __uint_as_float(bits << 16);
}

template <typename DT>
__device__ __forceinline__ void store_elem(void *row, int64_t e, float v)
{
    if constexpr (DT::kBytes == 4) reinterpret_cast<float *>(row)[e] = v;
    else reinterpret_cast<uint16_t *>(row)[e] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xFFFFu);
}

// non-temporal 16-byte row accesses: every byte of a logit row is touched exactly once
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

// ---- (max, sum) pairs of an online log-sum-exp:  sum_j exp(z_j) = s * exp(m) ----------------
struct MaxSum {
    float m, s;
};

__device__ __forceinline__ MaxSum combine(MaxSum a, MaxSum b)
{
    const float m = fmaxf(a.m, b.m);
    MaxSum o;
    o.m = m;
    o.s = a.s * exp2_hw((a.m - m) * kLog2e) + b.s * exp2_hw((b.m - m) * kLog2e);
    return o;
}

__device__ __forceinline__ MaxSum wave_reduce(MaxSum v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        MaxSum o;
        o.m = __shfl_xor(v.m, off, kWave);
        o.s = __shfl_xor(v.s, off, kWave);
        v = combine(v, o);
    }
    return v;
}

// Folds DT::kPerVec elements into a thread's running (m, s).
template <int N>
__device__ __forceinline__ void fold(MaxSum &acc, const float *f)
{
    float vmax = f[0];
#pragma unroll
    for (int e = 1; e < N; ++e) vmax = fmaxf(vmax, f[e]);
    const float m_new = fmaxf(acc.m, vmax);
    // differences first, then the scaling by log2(e): (z - m) is exact or rounded relative to the difference
    // itself, so the exponent's error does not grow with the magnitude of the logits
    float s = acc.s * exp2_hw((acc.m - m_new) * kLog2e);
#pragma unroll
    for (int e = 0; e < N; ++e) s += exp2_hw((f[e] - m_new) * kLog2e);
    acc.m = m_new;
    acc.s = s;
}

// z floored at -1e30 by one unsigned minimum: negative floats order like their bit patterns, so
// anything below the floor (and -inf) becomes the floor; non-negative values pass unchanged.
// Keeps p * z = 0 for z = -inf (p = 0) instead of NaN.
__device__ __forceinline__ float finite_floor(float x)
{
    return __uint_as_float(min(__float_as_uint(x), 0xF149F2CAu));
}

// The same online reduction with a third running quantity u = sum_j exp(z_j - m) * z_j, from which
// the policy entropy follows as H = lse - u / s  (H = -sum p log p, log p_j = z_j - lse).
struct MaxSumU {
    float m, s, u;
};

__device__ __forceinline__ MaxSumU combine(MaxSumU a, MaxSumU b)
{
    const float m = fmaxf(a.m, b.m);
    const float fa = exp2_hw((a.m - m) * kLog2e), fb = exp2_hw((b.m - m) * kLog2e);
    MaxSumU o;
    o.m = m;
    o.s = a.s * fa + b.s * fb;
    o.u = a.u * fa + b.u * fb;
    return o;
}

__device__ __forceinline__ MaxSumU wave_reduce(MaxSumU v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        MaxSumU o;
        o.m = __shfl_xor(v.m, off, kWave);
        o.s = __shfl_xor(v.s, off, kWave);
        o.u = __shfl_xor(v.u, off, kWave);
        v = combine(v, o);
    }
    return v;
}

// z = -inf (padding lanes, or a masked vocabulary entry) has exp(z - m) = 0; flooring z keeps the
// product 0 instead of 0 * inf.
template <int N>
__device__ __forceinline__ void fold(MaxSumU &acc, const float *f)
{
    float vmax = f[0];
#pragma unroll
    for (int e = 1; e < N; ++e) vmax = fmaxf(vmax, f[e]);
    const float m_new = fmaxf(acc.m, vmax);
    const float scale = exp2_hw((acc.m - m_new) * kLog2e);
    float s = acc.s * scale, u = acc.u * scale;
#pragma unroll
    for (int e = 0; e < N; ++e) {
        const float ex = exp2_hw((f[e] - m_new) * kLog2e);
        s += ex;
        u = fmaf(ex, finite_floor(f[e]), u);
    }
    acc.m = m_new;
    acc.s = s;
    acc.u = u;
}

// accumulator of a row reduction: (m, s) alone, or with u when the entropy is wanted
template <bool ENT> struct RowAcc { using type = MaxSum; };
template <> struct RowAcc<true> { using type = MaxSumU; };
__device__ __forceinline__ void seed(MaxSum &a) { a.m = kNegFloor; a.s = 0.0f; }
__device__ __forceinline__ void seed(MaxSumU &a) { a.m = kNegFloor; a.s = 0.0f; a.u = 0.0f; }
__device__ __forceinline__ float entropy_of(const MaxSum &, float) { return 0.0f; }
__device__ __forceinline__ float entropy_of(const MaxSumU &a, float lse) { return lse - a.u / a.s; }

// block-wide all-reduce of a row accumulator through LDS, two barriers; for the multi-pass kernels.
// `red` holds 3 * WAVES floats.
__device__ __forceinline__ void put(float *red, int waves, int w, const MaxSum &v)
{
    red[w] = v.m;
    red[waves + w] = v.s;
}
__device__ __forceinline__ void put(float *red, int waves, int w, const MaxSumU &v)
{
    red[w] = v.m;
    red[waves + w] = v.s;
    red[2 * waves + w] = v.u;
}
__device__ __forceinline__ void get(const float *red, int waves, int w, MaxSum &v)
{
    v.m = red[w];
    v.s = red[waves + w];
}
__device__ __forceinline__ void get(const float *red, int waves, int w, MaxSumU &v)
{
    v.m = red[w];
    v.s = red[waves + w];
    v.u = red[2 * waves + w];
}

template <int WAVES, typename ACC>
__device__ __forceinline__ ACC block_allreduce(ACC v, float *red)
{
    v = wave_reduce(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    __syncthreads();  // previous readers of red are done
    if (lane == 0) put(red, WAVES, wave, v);
    __syncthreads();
    ACC t;
    get(red, WAVES, 0, t);
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
        ACC o;
        get(red, WAVES, w, o);
        t = combine(t, o);
    }
    return t;
}

// ---- per-token A-3PO terms (Eq. 2 - Eq. 4 of the paper) -----------------------------------
struct TokenTerms {
    float alpha, lp, iw, r, obj, g;
    bool clipped, negative_staleness;
};

// lt = log pi_theta, lb = log pi_behav.  inv_n = 1/N (0 when N == 0).
// The ratios use the closed form of Section 3.1 (r = w^alpha, iw = w^(1-alpha), w = exp(lt-lb)),
// which is algebraically the same as exp(lt - lp), exp(lp - lb) without the cancellation.
// prox_mode: A3PO_PROX_INTERP (the paper's method, Eq. 3/4), A3PO_PROX_GIVEN (the proximal
// log-prob was computed by the caller - the "recompute" baseline of Section 4.2; `version` then
// carries its float bits), A3PO_PROX_BEHAV (proximal = behaviour policy: the coupled objective
// of Eq. 1, the "sync" baseline).
__device__ __forceinline__ TokenTerms token_terms(float lt, float lb, int32_t version, int32_t current_version,
                                                  float A, float clip_eps, float inv_n, int prox_mode)
{
    TokenTerms o;
    if (prox_mode == A3PO_PROX_GIVEN) {
        o.negative_staleness = false;
        o.alpha = 0.0f;
        o.lp = __int_as_float(version);
        o.r = expf(lt - o.lp);
        o.iw = expf(o.lp - lb);
    } else {
        const int64_t d = prox_mode == A3PO_PROX_BEHAV ? 0 : (int64_t)current_version - (int64_t)version;
        o.negative_staleness = d < 0;
        o.alpha = d >= 1 ? 1.0f / (float)d : 1.0f;
        const float one_minus = 1.0f - o.alpha;
        o.lp = o.alpha * lb + one_minus * lt;
        const float delta = lt - lb;
        o.r = expf(o.alpha * delta);
        o.iw = expf(one_minus * delta);
    }
    const float s1 = o.r * A;
    const float rc = fminf(fmaxf(o.r, 1.0f - clip_eps), 1.0f + clip_eps);
    const float s2 = rc * A;
    o.clipped = s2 < s1;
    o.obj = o.iw * (o.clipped ? s2 : s1);
    o.g = o.clipped ? 0.0f : -inv_n * o.iw * A * o.r;
    return o;
}

// flag bits stored per token in the workspace
enum : uint8_t { kFlagCounted = 1, kFlagClipped = 2, kFlagNegStale = 4 };

// Per-token inputs packed by the prep kernel so that the row kernel fetches them with one
// 16-byte scalar load.  y = -1 marks a token that does not enter the loss (masked, or a
// chosen id outside the vocabulary).
struct alignas(16) TokenRecord {
    int32_t y, ver;
    float lb, A;
};

// Per-token outputs of a vocabulary-wide loss kernel (logp / ent only where that kernel produces them).
struct RowOutputs {
    float *logp, *prox, *obj, *iw, *ent;
    uint8_t *flags;
};

// Workspace header written by the prep kernel, read by the row kernel and the finish kernel.
struct WsHeader {
    float inv_n;        // 1/N, or 0 when N == 0
    float n_as_float;   // N
    int64_t n_counted;  // tokens with mask != 0 and a valid id
    int64_t n_bad;      // tokens with mask != 0 and an invalid id
};

constexpr size_t kWsHeaderBytes = 256;
// The row kernel's work-queue counter lives in the header block, away from the read-only fields.
constexpr size_t kWsRowQueueOffset = 128;
__host__ __device__ inline unsigned int *row_queue_of(void *ws_header)
{
    return reinterpret_cast<unsigned int *>(static_cast<char *>(ws_header) + kWsRowQueueOffset);
}

}  // namespace a3po
