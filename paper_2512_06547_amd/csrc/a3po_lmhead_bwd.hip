// A-3PO loss forward + backward starting from hidden states and the LM-head weight.
//
// Only tokens that enter the loss (mask != 0 and a valid chosen id) are projected at all: every other token has
// log-prob 0 by definition and contributes nothing to the loss or to either gradient, so its hidden row never
// reaches the matrix cores.  The counted tokens are compacted on the device (an index of their positions, their
// hidden rows gathered into a dense matrix); how many there are is known only on the device, so every launch
// below is sized for the worst case and reads the count from memory - nothing waits for the host.
//
// The compacted tokens are processed in chunks.  For each chunk
//   1. z = h_chunk W^T on the matrix cores; every 256 x 256 tile is folded into the running (max, sum) of its
//      tokens while it is still in the accumulators (fp32: the log-sum-exp and the log-probs never see a rounded
//      logit) and is also stored, as fp32, for the backward pass of the same chunk;
//   2. log pi_theta, then Eq. 2 - Eq. 4 per token: loss terms, statistics and g_t = d loss / d log pi_theta;
//   3. dz[t, v] = g_t ([v == y_t] - exp(z[t, v] - lse_t)), rounded once to bfloat16 (the matrix cores take
//      bfloat16 operands), written token-major and vocabulary-major in one pass over the stored logits;
//   4. dh_chunk = dz W            (contraction over the vocabulary: dz token-major against W^T)
// and once per group of kLmDwGroup chunks
//   5. dW     += dz^T h_group     (contraction over the tokens: h^T against dz vocabulary-major; written in
//      bfloat16 straight from the accumulators when one group holds every token, else summed in an fp32
//      accumulator across groups and rounded to bfloat16 once at the end).
// All three contractions are the kernel of a3po_gemm.hip, which wants the contracted index contiguous in both
// operands; W^T and h^T are therefore written once per call.  6 N V H flops per step for N counted tokens: the
// logits of a chunk are kept (4 bytes each, 5 GB for 8,192 tokens at V = 151,936) rather than recomputed, which
// would be a fourth contraction.  Finally the rows of dh are scattered back to their tokens.
#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

#ifndef A3PO_LM_BWD_CHUNK
#define A3PO_LM_BWD_CHUNK 8192
#endif
constexpr int64_t kLmBwdChunk = A3PO_LM_BWD_CHUNK;  // tokens whose logits live in HBM at a time
// The weight gradient is contracted once per this many chunks: every contraction into it ends with a pass over the
// whole V x H accumulator, so fewer, longer ones are cheaper; the price is the vocabulary-major gradient of a
// whole group in memory (20 GB for 65,536 tokens at V = 151,936; batches up to that size need a single contraction and no
// accumulation pass at all).
constexpr int64_t kLmDwGroup = 8;
constexpr int64_t kPadK = 128;                      // contracted extents are zero-padded to this

struct LmBwdLayout {
    size_t lse, g, logp, ysel, index, pos, counts, partial, zt, dzt, dz, wt, hc, ht, dhc, dwacc, total;
    int64_t chunk;  // compacted tokens per chunk
    int64_t ldg;    // K extent of the vocabulary-major gradient: the tokens of a group of chunks, padded to kPadK
    int64_t ldv;    // K extent of the token-major gradient chunk and of W^T (and row stride of the chunk's logits): V padded
    int64_t ldt;    // K extent of h^T: T padded to kPadK
};

constexpr int kCompactBlock = 1024;  // tokens per workgroup of the compaction kernels

static LmBwdLayout lmhead_bwd_layout(int64_t T, int64_t V, int64_t H)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    auto pad = [](int64_t x) { return (x + kPadK - 1) / kPadK * kPadK; };
    const size_t t = (size_t)(T > 0 ? T : 0), v = (size_t)V, h = (size_t)H;
    LmBwdLayout l;
    l.chunk = T < kLmBwdChunk ? (T > 0 ? T : 1) : kLmBwdChunk;
    l.ldg = pad(T < kLmDwGroup * kLmBwdChunk ? (T > 0 ? T : 1) : kLmDwGroup * kLmBwdChunk);
    l.ldv = pad(V);
    l.ldt = pad(T > 0 ? T : 1);
    // per compacted token: lse, g, log pi, chosen id, position of the token; per token: its compacted position
    l.lse = up(loss_ws_layout(T).total);
    l.g = l.lse + up(t * sizeof(float));
    l.logp = l.g + up(t * sizeof(float));
    l.ysel = l.logp + up(t * sizeof(float));
    l.index = l.ysel + up(t * sizeof(int32_t));
    l.pos = l.index + up(t * sizeof(int32_t));
    l.counts = l.pos + up(t * sizeof(int32_t));
    l.partial = l.counts + up(((t + kCompactBlock - 1) / kCompactBlock + 1) * sizeof(int32_t));
    l.zt = l.partial + up((size_t)kGemmMaxPartialSlots * (size_t)l.chunk * sizeof(float2));
    l.dzt = l.zt + up((size_t)l.chunk * (size_t)l.ldv * sizeof(float));
    // the four operands that this file's own kernels write are kept in the contraction kernel's panel layout
    l.dz = l.dzt + up(panel_elements(V, l.ldg) * 2);
    l.wt = l.dz + up(panel_elements(l.chunk, l.ldv) * 2);
    l.hc = l.wt + up(panel_elements(H, l.ldv) * 2);
    l.ht = l.hc + up(t * h * 2);
    l.dhc = l.ht + up(panel_elements(H, l.ldt) * 2);
    l.dwacc = l.dhc + up(t * h * 2);
    // (the fp32 accumulator of dW exists only when the tokens may need more than one contraction)
    l.total = l.dwacc + (T > kLmDwGroup * kLmBwdChunk ? up(v * h * sizeof(float)) : 0);
    return l;
}

size_t lmhead_bwd_workspace_bytes(int64_t T, int64_t V, int64_t H) { return lmhead_bwd_layout(T, V, H).total; }

// dst = src rounded to bfloat16, or zeros when no token was counted (src was then never written)
__global__ void f32_to_bf16_kernel(const float *__restrict__ src, uint16_t *__restrict__ dst, size_t n,
                                   const int64_t *__restrict__ n_counted)
{
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 2;
    const bool any = *n_counted > 0;
    if (i + 1 < n) {
        *reinterpret_cast<uint32_t *>(dst + i) = any ? pack_bf16x2(src[i], src[i + 1]) : 0u;
    } else if (i < n) {
        dst[i] = any ? (uint16_t)(pack_bf16x2(src[i], 0.0f) & 0xFFFFu) : (uint16_t)0;
    }
}

// dst = zeros when no token was counted (the weight-gradient contraction was then a no-op and wrote nothing)
// (a fixed, small grid that strides over dst: in the usual case every workgroup only looks at the count)
__global__ void zero_bf16_if_none_kernel(uint16_t *__restrict__ dst, size_t n, const int64_t *__restrict__ n_counted)
{
    if (*n_counted > 0) return;
    const size_t step = (size_t)gridDim.x * blockDim.x * 2;
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 2; i < n; i += step) {
        if (i + 1 < n) *reinterpret_cast<uint32_t *>(dst + i) = 0u;
        else dst[i] = 0;
    }
}

// (fill kernels rather than hipMemsetAsync, so that the call can be captured into a HIP graph)
__global__ void zero_bf16_kernel(uint16_t *__restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0;
}

// zeroes the contracted positions [k0, k1) of every row of a panel-layout operand with `rows` rows (a multiple of 256)
__global__ void zero_panel_columns_kernel(uint16_t *__restrict__ m, int64_t rows, int64_t kext, int64_t k0, int64_t k1)
{
    const int64_t w = k1 - k0;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * w) m[panel_offset(i / w, k0 + i % w, kext)] = 0;
}

// out = transpose of in [R, C] (row-major, contiguous, 2-byte elements; C a multiple of 8) as a panel-layout operand
// with C rows and K extent ldo (>= R, a multiple of 64); positions R .. ldo-1 of every row (the padding of the
// contracted index) are written as zeros.
// A workgroup moves a 64 x 64 tile through LDS: 16-byte loads along the columns, 16-byte stores along the rows.
constexpr int kTrTile = 64;
__global__ __launch_bounds__(256) void transpose_pad_bf16_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out,
                                                                 int64_t R, int64_t C, int64_t ldo,
                                                                 const int64_t *__restrict__ R_dev)
{
    if (R_dev) R = *R_dev;  // rows that exist (the rest of `in` is not read)
    __shared__ uint16_t tile[kTrTile][kTrTile + 2];  // [row][column], padded: column reads below spread over the banks
    const int64_t r0 = (int64_t)blockIdx.y * kTrTile, c0 = (int64_t)blockIdx.x * kTrTile;
    const int tid = threadIdx.x;
    // load: 64 rows x 8 vectors of 8 columns; thread -> (row = tid / 8 + 32 * pass, vector = tid % 8)
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = tid / 8 + 32 * pass, cv = (tid % 8) * 8;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (r0 + r < R && c0 + cv < C) v = *reinterpret_cast<const uint4 *>(in + (r0 + r) * C + c0 + cv);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tile[r][cv + 2 * e] = (uint16_t)(w[e] & 0xFFFFu);
            tile[r][cv + 2 * e + 1] = (uint16_t)(w[e] >> 16);
        }
    }
    __syncthreads();
    // store: 64 columns x 8 vectors of 8 rows; thread -> (column = tid / 8 + 32 * pass, vector = tid % 8)
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = tid / 8 + 32 * pass, rv = (tid % 8) * 8;
        if (c0 + c >= C || r0 + rv >= ldo) continue;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)tile[rv + 2 * e][c] | ((uint32_t)tile[rv + 2 * e + 1][c] << 16);
        *reinterpret_cast<uint4 *>(out + panel_offset(c0 + c, r0 + rv, ldo)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

static hipError_t launch_transpose_pad(const uint16_t *in, uint16_t *out, int64_t R, int64_t C, int64_t ldo,
                                       const int64_t *R_dev, hipStream_t s)
{
    const dim3 grid((unsigned)((C + kTrTile - 1) / kTrTile), (unsigned)((ldo + kTrTile - 1) / kTrTile));
    hipLaunchKernelGGL(transpose_pad_bf16_kernel, grid, dim3(256), 0, s, in, out, R, C, ldo, R_dev);
    return hipGetLastError();
}

// ---- compaction of the counted tokens ----------------------------------------------------------------
// counts[b] = counted tokens among tokens [b, b + 1) * kCompactBlock (a record with y >= 0 is a counted token)
__global__ __launch_bounds__(256) void compact_count_kernel(const TokenRecord *__restrict__ records, int64_t T,
                                                            int32_t *__restrict__ counts)
{
    __shared__ int s_cnt[4];
    const int64_t t0 = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) c += (t0 + i < T && records[t0 + i].y >= 0) ? 1 : 0;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) c += __shfl_xor(c, off, kWave);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) counts[blockIdx.x] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
}

// Positions: counted token t gets the compacted position pos[t] = number of counted tokens before it, and
// index[pos] = t, ysel[pos] = its chosen id.  Tokens that are not counted get pos = -1 and their per-token
// outputs (zeros) here, since no later kernel visits them.
__global__ __launch_bounds__(256) void compact_index_kernel(const TokenRecord *__restrict__ records, int64_t T,
                                                            const int32_t *__restrict__ counts,
                                                            int32_t *__restrict__ index, int32_t *__restrict__ pos,
                                                            int32_t *__restrict__ ysel, float *logp, float *prox,
                                                            float *obj, float *iw, uint8_t *flags)
{
    __shared__ int s_part[4], s_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // counted tokens in the blocks before this one
    int before = 0;
    for (int b = tid; b < (int)blockIdx.x; b += 256) before += counts[b];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) before += __shfl_xor(before, off, kWave);
    if (lane == 0) s_part[wave] = before;
    __syncthreads();
    if (tid == 0) s_base = s_part[0] + s_part[1] + s_part[2] + s_part[3];
    __syncthreads();
    // this thread's four tokens, then an exclusive scan of the threads' counts over the workgroup
    const int64_t t0 = (int64_t)blockIdx.x * kCompactBlock + tid * 4;
    int y[4], c = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        y[i] = t0 + i < T ? records[t0 + i].y : -1;
        c += y[i] >= 0 ? 1 : 0;
    }
    int incl = c;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    __syncthreads();  // s_part is reused
    if (lane == kWave - 1) s_part[wave] = incl;
    __syncthreads();
    int at = s_base + incl - c;
    for (int w = 0; w < wave; ++w) at += s_part[w];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t t = t0 + i;
        if (t >= T) break;
        if (y[i] >= 0) {
            pos[t] = at;
            index[at] = (int32_t)t;
            ysel[at] = y[i];
            ++at;
        } else {
            pos[t] = -1;
            logp[t] = 0.0f;
            if (prox) prox[t] = 0.0f;
            obj[t] = 0.0f;
            iw[t] = 0.0f;
            flags[t] = 0;
        }
    }
}

// dst[j, :] = src[index[j], :] for j < *n (rows of C 2-byte elements, C a multiple of 8); one wavefront per row
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                          const int32_t *__restrict__ index, const int64_t *__restrict__ n,
                                                          int64_t C)
{
    const int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= *n) return;
    const uint16_t *from = src + (int64_t)index[j] * C;
    uint16_t *to = dst + j * C;
    for (int64_t k = (int64_t)(threadIdx.x & 63) * 8; k < C; k += 64 * 8)
        *reinterpret_cast<uint4 *>(to + k) = *reinterpret_cast<const uint4 *>(from + k);
}

// dst[t, :] = src[pos[t], :] where pos[t] >= 0, zeros elsewhere (every row of dst is written)
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                           const int32_t *__restrict__ pos, int64_t T, int64_t C)
{
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int32_t p = pos[t];
    uint16_t *to = dst + t * C;
    for (int64_t k = (int64_t)(threadIdx.x & 63) * 8; k < C; k += 64 * 8)
        *reinterpret_cast<uint4 *>(to + k) =
            p >= 0 ? *reinterpret_cast<const uint4 *>(src + (int64_t)p * C + k) : make_uint4(0u, 0u, 0u, 0u);
}

// Per-token terms of a chunk of compacted tokens once their log-probs are known (Eq. 2 - Eq. 4): what the fused
// row kernel does for logits that come from memory.  Compacted token j of the chunk is token index[j]; its
// outputs go to that token's place, g stays in compacted order for the gradient kernel.
__global__ void lmhead_token_terms_kernel(const TokenRecord *__restrict__ records, const int32_t *__restrict__ index,
                                          DynCount count, int32_t current_version, float clip_eps,
                                          const WsHeader *__restrict__ hdr, const float *__restrict__ logp_c,
                                          float *logp, float *prox, float *obj, float *iw, uint8_t *flags,
                                          float *g_out)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= dyn_extent(count, 0)) return;
    const int64_t t = index[j];
    const TokenRecord rec = records[t];
    const float lt = logp_c[j];
    const TokenTerms tt = token_terms(lt, rec.lb, rec.ver, current_version, rec.A, clip_eps, hdr->inv_n, A3PO_PROX_INTERP);
    logp[t] = lt;
    if (prox) prox[t] = tt.lp;
    obj[t] = tt.obj;
    iw[t] = tt.iw;
    flags[t] = (uint8_t)(kFlagCounted | (tt.clipped ? kFlagClipped : 0) | (tt.negative_staleness ? kFlagNegStale : 0));
    g_out[j] = tt.g;
}

// Gradient of a chunk's logits from the stored fp32 logits z [n, ldv] (token-major):
//   dz[t, v] = g_t ([v == y_t] - exp(z[t, v] - lse_t)),
// rounded once to bfloat16 and written both token-major (dz: n rows, K extent ldv; the operand of the hidden-state
// gradient) and vocabulary-major (dzt: V rows, K extent ldg, at token position col0; the operand of the weight
// gradient), both in the contraction kernel's panel layout, in which a 64 x 64 tile is two runs of 4 KiB.  A workgroup takes
// a tile of 64 tokens x 64 vocabulary entries: 16-byte loads and 8-byte stores along the vocabulary, then through
// LDS 16-byte stores along the tokens.  Token columns n .. (next multiple of 128) of dzt are written as zeros (they
// pad the contraction over the tokens); a token with g = 0 gives an exactly zero row.  lse, g, ysel: the chunk's
// tokens in compacted order.
constexpr int kDzTile = 64;
__global__ __launch_bounds__(256) void lmhead_dz_kernel(const float *__restrict__ zc, int64_t V, DynCount count, int64_t ldv,
                                                        const float *__restrict__ lse, const float *__restrict__ g,
                                                        const int32_t *__restrict__ ysel, uint16_t *__restrict__ dz,
                                                        uint16_t *__restrict__ dzt, int64_t ldg, int64_t col0)
{
    __shared__ __align__(16) uint16_t tile[kDzTile][kDzTile + 8];  // [vocabulary entry][token], rows 144 bytes apart
    const int tid = threadIdx.x;
    const int64_t n = dyn_extent(count, 0);
    const int64_t v0 = (int64_t)blockIdx.x * kDzTile, t0 = (int64_t)blockIdx.y * kDzTile;
    if (t0 >= (n + kPadK - 1) / kPadK * kPadK) return;  // past the padded chunk (uniform)
    const int vq = (tid & 15) * 4;  // this thread's four vocabulary entries: v0 + vq ..
    const int64_t v = v0 + vq;      // (V and vq are multiples of 4: the four are inside or outside as a whole)
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int tr = (tid >> 4) + 16 * pass;
        const int64_t t = t0 + tr;
        float d[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (t < n && v < V) {
            const float neg_g = -g[t];
            if (neg_g != 0.0f) {
                const float tl = lse[t];
                const int64_t y = ysel[t];
                const float4 z = *reinterpret_cast<const float4 *>(zc + t * ldv + v);
                const float zz[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = exp2_hw((zz[i] - tl) * kLog2e);
                    d[i] = neg_g * p - (y == v + i ? neg_g : 0.0f);
                }
            }
        }
        const uint32_t lo = pack_bf16x2(d[0], d[1]), hi = pack_bf16x2(d[2], d[3]);
        if (t < n && v < V) *reinterpret_cast<uint2 *>(dz + panel_offset(t, v, ldv)) = make_uint2(lo, hi);
        tile[vq + 0][tr] = (uint16_t)(lo & 0xFFFFu);
        tile[vq + 1][tr] = (uint16_t)(lo >> 16);
        tile[vq + 2][tr] = (uint16_t)(hi & 0xFFFFu);
        tile[vq + 3][tr] = (uint16_t)(hi >> 16);
    }
    __syncthreads();
    // vocabulary-major: 64 entries x 2 panel blocks of 32 tokens; thread -> entry tid / 4, 8 tokens of each block, so
    // that the four lanes of an entry write 64 contiguous bytes and a wavefront 1 KiB per store instruction
    const int vr = tid >> 2, tq = (tid & 3) * 8;
    if (v0 + vr < V) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const uint4 w = *reinterpret_cast<const uint4 *>(&tile[vr][32 * half + tq]);
            *reinterpret_cast<uint4 *>(dzt + panel_offset(v0 + vr, col0 + t0 + 32 * half + tq, ldg)) = w;
        }
    }
}

}  // namespace a3po

using namespace a3po;

extern "C" int a3po_fused_lmhead_loss_fwd_bwd(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                              const int32_t *chosen, const float *logp_behav, const int32_t *versions,
                                              int32_t current_version, const float *advantages,
                                              const uint8_t *loss_mask, float clip_eps, float denom, void *dhidden,
                                              void *dweight, float *logp_out, float *logp_prox_out, float *loss_out,
                                              a3po_stats *stats_out, void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    auto aligned = [](const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; };
    // H <= 2^20 and V < 2^21 keep the contraction kernel's 32-bit byte offsets inside a 256-row tile below 2^32
    // (and T < 2^22: a row of h^T is T elements long)
    if (T < 0 || V <= 0 || H <= 0 || H % 64 != 0 || H > (1 << 20) || V % 8 != 0 || V > (1 << 21) - 128 || T > (1 << 22) - 128)
        return A3PO_E_SIZE;
    if (!(clip_eps >= 0.0f && clip_eps < 1.0f) || denom != denom) return A3PO_E_VALUE;
    if (!loss_out || !weight || !dweight) return A3PO_E_NULL;
    if (T > 0 && (!hidden || !dhidden || !chosen || !logp_behav || !versions || !advantages || !loss_mask || !logp_out))
        return A3PO_E_NULL;
    if (!aligned(hidden, 16) || !aligned(weight, 16) || !aligned(dhidden, 16) || !aligned(dweight, 16))
        return A3PO_E_ALIGN;
    const LmBwdLayout lay = lmhead_bwd_layout(T, V, H);
    if (!workspace || workspace_bytes < lay.total) return A3PO_E_WORKSPACE;
    if (!aligned(workspace, 256)) return A3PO_E_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *lse = reinterpret_cast<float *>(ws + lay.lse);        // the next four: compacted order
    float *gtok = reinterpret_cast<float *>(ws + lay.g);
    float *logp_c = reinterpret_cast<float *>(ws + lay.logp);
    int32_t *ysel = reinterpret_cast<int32_t *>(ws + lay.ysel);
    int32_t *index = reinterpret_cast<int32_t *>(ws + lay.index);  // compacted position -> token
    int32_t *pos = reinterpret_cast<int32_t *>(ws + lay.pos);      // token -> compacted position or -1
    int32_t *counts = reinterpret_cast<int32_t *>(ws + lay.counts);
    float2 *partial = reinterpret_cast<float2 *>(ws + lay.partial);
    float *zt = reinterpret_cast<float *>(ws + lay.zt);            // the chunk's logits [chunk, ldv], fp32
    uint16_t *dzt = reinterpret_cast<uint16_t *>(ws + lay.dzt);
    uint16_t *dz = reinterpret_cast<uint16_t *>(ws + lay.dz);
    uint16_t *wt = reinterpret_cast<uint16_t *>(ws + lay.wt);
    uint16_t *hc = reinterpret_cast<uint16_t *>(ws + lay.hc);      // hidden rows of the counted tokens
    uint16_t *ht = reinterpret_cast<uint16_t *>(ws + lay.ht);      // and their transpose
    uint16_t *dhc = reinterpret_cast<uint16_t *>(ws + lay.dhc);
    float *dwacc = reinterpret_cast<float *>(ws + lay.dwacc);
    const uint16_t *h = static_cast<const uint16_t *>(hidden);
    const uint16_t *W = static_cast<const uint16_t *>(weight);
    const size_t nw = (size_t)V * (size_t)H;
    // up to kLmDwGroup chunks of tokens: a single weight-gradient contraction, which stores dW in bfloat16 itself
    const bool single_group = T <= kLmDwGroup * kLmBwdChunk;

    LossArgs a;
    a.z = nullptr;
    a.dz = nullptr;
    a.dt = A3PO_BF16;
    a.T = T;
    a.V = V;
    a.ld = V;
    a.chosen = chosen;
    a.lb = logp_behav;
    a.versions = versions;
    a.current_version = current_version;
    a.adv = advantages;
    a.mask = loss_mask;
    a.clip_eps = clip_eps;
    a.denom = denom;
    a.logp_out = logp_out;
    a.prox_out = logp_prox_out;
    a.loss_out = loss_out;
    a.stats_out = stats_out;
    carve_loss_ws(a, ws, T);
    const WsHeader *hdr = reinterpret_cast<const WsHeader *>(a.ws_header);
    const int64_t *n_counted = &hdr->n_counted;  // device: known once the prep kernel has run

    // token count, 1/N and the per-token records for the whole batch
    if (launch_loss_prep(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (T == 0) {
        if (launch_loss_finish(a, s) != hipSuccess) return A3PO_E_LAUNCH;
        hipLaunchKernelGGL(zero_bf16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s,
                           static_cast<uint16_t *>(dweight), nw);
        return hipGetLastError() == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
    }
    // compaction of the counted tokens, their hidden rows, and the transposed operands of the two backward
    // contractions (padding of the contracted index zeroed)
    const unsigned cblocks = (unsigned)((T + kCompactBlock - 1) / kCompactBlock);
    hipLaunchKernelGGL(compact_count_kernel, dim3(cblocks), dim3(256), 0, s, a.ws_records, T, counts);
    hipLaunchKernelGGL(compact_index_kernel, dim3(cblocks), dim3(256), 0, s, a.ws_records, T, counts, index, pos, ysel,
                       logp_out, logp_prox_out, a.ws_obj, a.ws_iw, a.ws_flags);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s, h, hc, index, n_counted, H);
    if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
    if (launch_transpose_pad(W, wt, V, H, lay.ldv, nullptr, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (launch_transpose_pad(hc, ht, T, H, lay.ldt, n_counted, s) != hipSuccess) return A3PO_E_LAUNCH;
    if (lay.ldv > V) {  // padding of the contracted index in the token-major gradient chunk: never written below
        const int64_t rows = (lay.chunk + 255) / 256 * 256, cells = rows * (lay.ldv - V);
        hipLaunchKernelGGL(zero_panel_columns_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, s, dz, rows,
                           lay.ldv, V, lay.ldv);
        if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
    }

    // Chunks of compacted tokens.  The host only knows the upper bound T; a chunk that starts past the counted
    // tokens finds an extent of zero on the device and its launches return at once.
    for (int64_t c0 = 0; c0 < T; c0 += lay.chunk) {
        const int64_t nmax = T - c0 < lay.chunk ? T - c0 : lay.chunk;
        const int64_t kmax = (nmax + kPadK - 1) / kPadK * kPadK;
        DynCount cnt;
        cnt.n = n_counted;
        cnt.offset = c0;
        cnt.cap = nmax;
        // 1. z [n, V] = h_chunk W^T (vocabulary on the row side of the tiles, stored transposed), folded into
        //    (max, sum) per token on the way out
        GemmArgs fw = {};
        fw.A = W;
        fw.lda = H;
        fw.B = hc + c0 * H;
        fw.ldb = H;
        fw.M = V;
        fw.N = nmax;
        fw.K = H;
        fw.C = zt;
        fw.ldc = lay.ldv;
        fw.transposed = 1;
        fw.partial = partial;
        fw.partial_stride = lay.chunk;
        fw.dyn_dim = kDynN;
        fw.dyn = cnt;
        if (launch_gemm_nt(fw, kEpiLseStore, s) != hipSuccess) return A3PO_E_LAUNCH;
        // 2. log pi_theta and the per-token terms
        if (launch_lmhead_lse_finish(hc + c0 * H, W, nmax, H, V, ysel + c0, partial, lay.chunk, logp_c + c0, lse + c0, s,
                                     cnt) != hipSuccess)
            return A3PO_E_LAUNCH;
        hipLaunchKernelGGL(lmhead_token_terms_kernel, dim3((unsigned)((nmax + 255) / 256)), dim3(256), 0, s,
                           a.ws_records, index + c0, cnt, current_version, clip_eps, hdr, logp_c + c0, logp_out,
                           logp_prox_out, a.ws_obj, a.ws_iw, a.ws_flags, gtok + c0);
        if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
        // 3. the gradient chunk in both layouts
        const int64_t g0 = c0 / (kLmDwGroup * lay.chunk) * (kLmDwGroup * lay.chunk);  // first token of this chunk's group
        const dim3 dz_grid((unsigned)((V + kDzTile - 1) / kDzTile), (unsigned)(kmax / kDzTile));
        hipLaunchKernelGGL(lmhead_dz_kernel, dz_grid, dim3(256), 0, s, zt, V, cnt, lay.ldv, lse + c0, gtok + c0,
                           ysel + c0, dz, dzt, lay.ldg, c0 - g0);
        if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
        // 4. dh_chunk [n, H] = dz [n, V] (W^T [H, V])^T
        GemmArgs bh = {};
        bh.A = dz;
        bh.lda = lay.ldv;
        bh.a_panel = 1;
        bh.B = wt;
        bh.ldb = lay.ldv;
        bh.b_panel = 1;
        bh.M = nmax;
        bh.N = H;
        bh.K = lay.ldv;
        bh.C = dhc + c0 * H;
        bh.ldc = H;
        bh.dyn_dim = kDynM;
        bh.dyn = cnt;
        if (launch_gemm_nt(bh, kEpiStoreBf16, s) != hipSuccess) return A3PO_E_LAUNCH;
        // 5. at the end of a group of chunks: dW [V, H] += (dz^T [V, group] (h^T [H, group])^T): h^T on the row side
        //    of the tiles, stored transposed; fp32 accumulator across groups
        const bool group_ends = c0 + lay.chunk >= T || (c0 + lay.chunk) % (kLmDwGroup * lay.chunk) == 0;
        if (group_ends) {
            const int64_t gmax = c0 + nmax - g0;  // tokens of the group, at most
            DynCount gcnt;
            gcnt.n = n_counted;
            gcnt.offset = g0;
            gcnt.cap = gmax;
            GemmArgs bw = {};
            bw.A = ht + panel_offset(0, g0, lay.ldt);
            bw.lda = lay.ldt;
            bw.a_panel = 1;
            bw.B = dzt;
            bw.ldb = lay.ldg;
            bw.b_panel = 1;
            bw.M = H;
            bw.N = V;
            bw.K = (gmax + kPadK - 1) / kPadK * kPadK;
            bw.C = single_group ? dweight : static_cast<void *>(dwacc);
            bw.ldc = H;
            bw.transposed = 1;
            bw.accumulate = g0 > 0;
            bw.dyn_dim = kDynK;
            bw.dyn = gcnt;
            if (launch_gemm_nt(bw, single_group ? kEpiStoreBf16 : kEpiAccumF32, s) != hipSuccess) return A3PO_E_LAUNCH;
        }
    }
    if (launch_loss_finish(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s, dhc,
                       static_cast<uint16_t *>(dhidden), pos, T, H);
    if (single_group)
        hipLaunchKernelGGL(zero_bf16_if_none_kernel, dim3((unsigned)(nw / 512 < 2048 ? nw / 512 + 1 : 2048)), dim3(256), 0, s,
                           static_cast<uint16_t *>(dweight), nw, n_counted);
    else
        hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((nw / 2 + 255) / 256)), dim3(256), 0, s, dwacc,
                           static_cast<uint16_t *>(dweight), nw, n_counted);
    return hipGetLastError() == hipSuccess ? A3PO_OK : A3PO_E_LAUNCH;
}
