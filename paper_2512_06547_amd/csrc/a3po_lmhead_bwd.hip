// A-3PO loss forward + backward starting from hidden states and the LM-head weight.
//
// The logits of a chunk of tokens are materialised in bfloat16 (chunk x V), run through the fused
// row kernel in place (log-softmax, proximal interpolation, clipped surrogate, gradient rows), and
// the gradient chunk is contracted back:  dh = dz W  and  dW += dz^T h.  With 288 GB of HBM a
// chunk of 8,192 tokens (2.5 GB at V = 151,936) is small change, so the projection is computed
// once (6 T V H flops in total) instead of being recomputed for the backward pass.
//
// The three contractions are plain GEMMs and go to rocBLAS (bfloat16 in, fp32 accumulate); dW is
// accumulated across chunks in fp32 and rounded to bfloat16 once at the end.  Everything between
// the GEMMs is this library's own kernels.
//
// dW = dz^T h contracts over the tokens, which is the slow dimension of both dz [n, V] and h [n, H] as they
// lie in memory; the matrix cores want the contracted index contiguous.  The gradient chunk and the hidden
// chunk are therefore transposed once (dzT [V, n], hT [H, n]; one more read and write of the chunk) and the
// product runs in the form with both operands contiguous along the tokens: 8.05 against 9.93 ms per chunk
// for the GEMM at the 8B shape, about 1 ms for the two transposes.
#include <mutex>

#include <rocblas/rocblas.h>

#include "a3po_common.h"
#include "a3po_launch.h"

namespace a3po {

#ifndef A3PO_LM_BWD_CHUNK
#define A3PO_LM_BWD_CHUNK 8192
#endif
constexpr int64_t kLmBwdChunk = A3PO_LM_BWD_CHUNK;  // tokens whose logits live in HBM at a time

struct LmBwdLayout {
    size_t loss_ws, zchunk, dzt, ht, dwacc, total;
    int64_t chunk;
    int64_t ldt;  // row stride of the transposed chunks: the chunk length rounded up to 8 tokens (16 bytes)
};

static LmBwdLayout lmhead_bwd_layout(int64_t T, int64_t V, int64_t H)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    LmBwdLayout l;
    l.chunk = T < kLmBwdChunk ? (T > 0 ? T : 1) : kLmBwdChunk;
    l.loss_ws = 0;
    l.ldt = (l.chunk + 7) / 8 * 8;
    l.zchunk = up(loss_ws_layout(T).total);
    l.dzt = l.zchunk + up((size_t)l.chunk * (size_t)V * 2);
    l.ht = l.dzt + up((size_t)V * (size_t)l.ldt * 2);
    l.dwacc = l.ht + up((size_t)H * (size_t)l.ldt * 2);
    l.total = l.dwacc + up((size_t)V * (size_t)H * sizeof(float));
    return l;
}

size_t lmhead_bwd_workspace_bytes(int64_t T, int64_t V, int64_t H) { return lmhead_bwd_layout(T, V, H).total; }

__global__ void f32_to_bf16_kernel(const float *__restrict__ src, uint16_t *__restrict__ dst, size_t n)
{
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 2;
    if (i + 1 < n) {
        *reinterpret_cast<uint32_t *>(dst + i) = pack_bf16x2(src[i], src[i + 1]);
    } else if (i < n) {
        dst[i] = (uint16_t)(pack_bf16x2(src[i], 0.0f) & 0xFFFFu);
    }
}

// (a fill kernel rather than hipMemsetAsync, so that the call can be captured into a HIP graph)
__global__ void zero_bf16_kernel(uint16_t *__restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0;
}

static rocblas_handle blas_handle()
{
    static rocblas_handle handle = nullptr;
    static std::once_flag once;
    std::call_once(once, [] {
        if (rocblas_create_handle(&handle) != rocblas_status_success) handle = nullptr;
    });
    return handle;
}

// out [C, ldo] = transpose of in [R, C] (row-major, 2-byte elements; C a multiple of 8, ldo >= R a multiple of 8).
// A workgroup moves a 64 x 64 tile through LDS: 16-byte loads along the columns, 16-byte stores along the rows.
// Rows beyond R inside the last 8-row group of a tile are stored as zeros (they lie in the padding of `out`).
constexpr int kTrTile = 64;
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out,
                                                             int64_t R, int64_t C, int64_t ldo)
{
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
        if (c0 + c >= C || r0 + rv >= R) continue;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)tile[rv + 2 * e][c] | ((uint32_t)tile[rv + 2 * e + 1][c] << 16);
        *reinterpret_cast<uint4 *>(out + (c0 + c) * ldo + r0 + rv) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

static hipError_t launch_transpose_bf16(const uint16_t *in, uint16_t *out, int64_t R, int64_t C, int64_t ldo, hipStream_t s)
{
    const dim3 grid((unsigned)((C + kTrTile - 1) / kTrTile), (unsigned)((R + kTrTile - 1) / kTrTile));
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, s, in, out, R, C, ldo);
    return hipGetLastError();
}

// column-major C[m,n] = alpha op(A) op(B) + beta C with bf16 A, B and fp32 accumulation
static bool gemm_bf16(rocblas_handle hd, rocblas_operation ta, rocblas_operation tb, int64_t m, int64_t n, int64_t k,
                      const void *A, int64_t lda, const void *B, int64_t ldb, float beta, void *C, int64_t ldc,
                      rocblas_datatype c_type)
{
    const float alpha = 1.0f;
    return rocblas_gemm_ex(hd, ta, tb, (rocblas_int)m, (rocblas_int)n, (rocblas_int)k, &alpha, A, rocblas_datatype_bf16_r,
                           (rocblas_int)lda, B, rocblas_datatype_bf16_r, (rocblas_int)ldb, &beta, C, c_type,
                           (rocblas_int)ldc, C, c_type, (rocblas_int)ldc, rocblas_datatype_f32_r,
                           rocblas_gemm_algo_standard, 0, 0) == rocblas_status_success;
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
    if (T < 0 || V <= 0 || H <= 0 || H % 8 != 0 || H > (1 << 20) || V % 8 != 0 || V > (int64_t)0x7FFFFFFF)
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
    rocblas_handle hd = blas_handle();
    if (!hd || rocblas_set_stream(hd, s) != rocblas_status_success) return A3PO_E_LAUNCH;
    if (rocblas_set_pointer_mode(hd, rocblas_pointer_mode_host) != rocblas_status_success) return A3PO_E_LAUNCH;

    char *ws = static_cast<char *>(workspace);
    uint16_t *zc = reinterpret_cast<uint16_t *>(ws + lay.zchunk);
    uint16_t *dzt = reinterpret_cast<uint16_t *>(ws + lay.dzt);
    uint16_t *ht = reinterpret_cast<uint16_t *>(ws + lay.ht);
    float *dwacc = reinterpret_cast<float *>(ws + lay.dwacc);
    const uint16_t *h = static_cast<const uint16_t *>(hidden);
    uint16_t *dh = static_cast<uint16_t *>(dhidden);

    LossArgs a;
    a.z = zc;
    a.dz = zc;
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

    // token count, 1/N and the per-token records for the whole batch
    if (launch_loss_prep(a, s) != hipSuccess) return A3PO_E_LAUNCH;

    for (int64_t c0 = 0; c0 < T; c0 += lay.chunk) {
        const int64_t n = T - c0 < lay.chunk ? T - c0 : lay.chunk;
        // logits of the chunk: z^T [V, n] = W [H, V]^T h_chunk [H, n]   (column-major views)
        if (!gemm_bf16(hd, rocblas_operation_transpose, rocblas_operation_none, V, n, H, weight, H, h + c0 * H, H, 0.0f,
                       zc, V, rocblas_datatype_bf16_r))
            return A3PO_E_LAUNCH;
        // loss forward + gradient rows over the chunk, in place
        LossArgs c = a;
        c.T = n;
        c.ws_records = a.ws_records + c0;
        c.logp_out = logp_out + c0;
        c.prox_out = logp_prox_out ? logp_prox_out + c0 : nullptr;
        c.ws_obj = a.ws_obj + c0;
        c.ws_iw = a.ws_iw + c0;
        c.ws_flags = a.ws_flags + c0;
        c.ws_lse = a.ws_lse + c0;
        c.ws_partial = a.ws_partial + c0;
        if (c0 > 0 && launch_reset_row_queue(ws, s) != hipSuccess) return A3PO_E_LAUNCH;
        if (launch_loss_rows(c, s) != hipSuccess) return A3PO_E_LAUNCH;
        // dh_chunk^T [H, n] = W [H, V] dz^T [V, n]
        if (!gemm_bf16(hd, rocblas_operation_none, rocblas_operation_none, H, n, V, weight, H, zc, V, 0.0f, dh + c0 * H,
                       H, rocblas_datatype_bf16_r))
            return A3PO_E_LAUNCH;
        // dW^T [H, V] += hT [n, H]^T dzT [n, V]       (column-major views of the transposed chunks, tokens
        // contiguous in both; fp32 accumulator across chunks)
        const int64_t ldt = (n + 7) / 8 * 8;
        if (launch_transpose_bf16(zc, dzt, n, V, ldt, s) != hipSuccess) return A3PO_E_LAUNCH;
        if (launch_transpose_bf16(h + c0 * H, ht, n, H, ldt, s) != hipSuccess) return A3PO_E_LAUNCH;
        if (!gemm_bf16(hd, rocblas_operation_transpose, rocblas_operation_none, H, V, n, ht, ldt, dzt, ldt,
                       c0 == 0 ? 0.0f : 1.0f, dwacc, H, rocblas_datatype_f32_r))
            return A3PO_E_LAUNCH;
    }
    if (launch_loss_finish(a, s) != hipSuccess) return A3PO_E_LAUNCH;
    const size_t nw = (size_t)V * (size_t)H;
    if (T == 0) {
        hipLaunchKernelGGL(zero_bf16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s,
                           static_cast<uint16_t *>(dweight), nw);
        if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
    } else {
        hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((nw / 2 + 255) / 256)), dim3(256), 0, s, dwacc,
                           static_cast<uint16_t *>(dweight), nw);
        if (hipGetLastError() != hipSuccess) return A3PO_E_LAUNCH;
    }
    return A3PO_OK;
}
