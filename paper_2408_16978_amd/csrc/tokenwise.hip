// Token-wise chunked neighbours of the attention path (Sec. 5.4): see include/fpdt_tokenwise.h.
// Library GEMMs (rocBLAS) for the dense products, a HIP kernel for the row-wise softmax / loss.
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <string>

#include "../../include/fpdt_tokenwise.h"

namespace {

enum { TW_OK = 0, TW_INVALID = 1, TW_UNSUPPORTED = 2, TW_WORKSPACE = 3, TW_HIP = 4 };

thread_local std::string g_err;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                            \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return fail(TW_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
#define BLAS_TRY(expr)                                                                            \
    do {                                                                                          \
        rocblas_status s_ = (expr);                                                               \
        if (s_ != rocblas_status_success)                                                         \
            return fail(TW_HIP, "%s failed: %s", #expr, rocblas_status_to_string(s_));            \
    } while (0)

std::mutex g_mu;
rocblas_handle g_handle = nullptr;

int get_handle(rocblas_handle* h, hipStream_t st)
{
    if (!g_handle) BLAS_TRY(rocblas_create_handle(&g_handle));
    BLAS_TRY(rocblas_set_stream(g_handle, st));
    BLAS_TRY(rocblas_set_pointer_mode(g_handle, rocblas_pointer_mode_host));
    *h = g_handle;
    return TW_OK;
}

// Row-major C[M,N] (+)= alpha * A[M,K] * B^T where B is [N,K]  ("NT": both operands K-contiguous),
// as the column-major product C^T[N,M] = B[N,K] ... expressed for rocBLAS:
//   C_cm[N x M, ld N] = op(B_cm)[N x K] * A_cm[K x M], B_cm = B^T stored [K x N, ld K] -> transA = T.
int gemm_nt(rocblas_handle h, int M, int N, int K, const void* A, const void* B, void* C,
            rocblas_datatype c_type, float beta)
{
    const float alpha = 1.f;
    BLAS_TRY(rocblas_gemm_ex(h, rocblas_operation_transpose, rocblas_operation_none, N, M, K, &alpha, B,
                             rocblas_datatype_bf16_r, K, A, rocblas_datatype_bf16_r, K, &beta, C, c_type, N, C,
                             c_type, N, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0));
    return TW_OK;
}
// Row-major C[M,N] = A[M,K] * B[K,N]  ("NN"): C_cm[N x M] = B_cm[N x K, ld N] * A_cm[K x M, ld K].
int gemm_nn(rocblas_handle h, int M, int N, int K, const void* A, const void* B, void* C,
            rocblas_datatype c_type, float beta)
{
    const float alpha = 1.f;
    BLAS_TRY(rocblas_gemm_ex(h, rocblas_operation_none, rocblas_operation_none, N, M, K, &alpha, B,
                             rocblas_datatype_bf16_r, N, A, rocblas_datatype_bf16_r, K, &beta, C, c_type, N, C,
                             c_type, N, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0));
    return TW_OK;
}
// Row-major C[M,N] (+)= A^T * B with A [K,M], B [K,N]  ("TN": contraction over rows):
//   C_cm[N x M] = B_cm[N x K, ld N] * (A_cm[M x K, ld M])^T.
int gemm_tn(rocblas_handle h, int M, int N, int K, const void* A, const void* B, void* C,
            rocblas_datatype c_type, float beta)
{
    const float alpha = 1.f;
    BLAS_TRY(rocblas_gemm_ex(h, rocblas_operation_none, rocblas_operation_transpose, N, M, K, &alpha, B,
                             rocblas_datatype_bf16_r, N, A, rocblas_datatype_bf16_r, M, &beta, C, c_type, N, C,
                             c_type, N, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0));
    return TW_OK;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}
__device__ __forceinline__ uint16_t to_bf16(float f)
{
    const unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);              // round to nearest even
}

// One workgroup per row of logits [n, vocab] fp32: lse, loss and (G != nullptr) the bf16
// gradient grad_scale * (softmax - onehot).  Two passes over the row: HBM-bound.
__global__ __launch_bounds__(256) void loss_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ target,
                                                        int vocab, float grad_scale, float* __restrict__ loss,
                                                        float* __restrict__ lse_out, uint16_t* __restrict__ G)
{
    __shared__ float red[2][4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const float* x = logits + (size_t)row * vocab;
    // running (max, sum of exp) per thread, merged across the workgroup
    float m = -INFINITY, l = 0.f;
    for (int v = tid; v < vocab; v += 256) {
        const float a = x[v];
        if (a > m) {
            l = l * __expf(m - a) + 1.f;
            m = a;
        } else {
            l += __expf(a - m);
        }
    }
    const float wm = wave_max(m);
    l = wave_sum(m == -INFINITY ? 0.f : l * __expf(m - wm));
    if (lane == 0) { red[0][w] = wm; red[1][w] = l; }
    __syncthreads();
    const float gm = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    float gl = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) gl += red[1][i] * __expf(red[0][i] - gm);
    const float lse = gm + __logf(gl);
    const int t = target[row];
    if (tid == 0) {
        lse_out[row] = lse;
        loss[row] = lse - ((t >= 0 && t < vocab) ? x[t] : 0.f);
    }
    if (!G) return;
    uint16_t* g = G + (size_t)row * vocab;
    for (int v = tid; v < vocab; v += 256) {
        const float p = __expf(x[v] - lse) - (v == t ? 1.f : 0.f);
        g[v] = to_bf16(grad_scale * p);
    }
}

}  // namespace

extern "C" {

size_t fpdt_tw_loss_workspace_bytes(int64_t rows, int hidden, int vocab, int n_chunks)
{
    if (rows <= 0 || hidden <= 0 || vocab <= 0 || n_chunks <= 0 || n_chunks > rows) return 0;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    const size_t logits = ((size_t)c * vocab * 4 + 255) & ~(size_t)255;
    const size_t grad = ((size_t)c * vocab * 2 + 255) & ~(size_t)255;
    return logits + grad;
}

int fpdt_tw_loss_fwd_bwd(const void* H, const void* W, const int32_t* target, float grad_scale, float* loss,
                         float* lse, void* dH, float* dW, int64_t rows, int hidden, int vocab, int n_chunks,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    g_err.clear();
    if (!H || !W || !target || !loss || !lse) return fail(TW_INVALID, "NULL tensor pointer");
    if (rows <= 0 || hidden <= 0 || vocab <= 0) return fail(TW_INVALID, "rows, hidden and vocab must be positive");
    if (n_chunks <= 0 || n_chunks > rows) return fail(TW_INVALID, "n_chunks=%d must be in [1, rows]", n_chunks);
    if (!std::isfinite(grad_scale)) return fail(TW_INVALID, "grad_scale must be finite");
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    if (c > (int64_t)1 << 24 || vocab > (1 << 24) || hidden > (1 << 20)) return fail(TW_UNSUPPORTED, "sizes beyond the 32-bit GEMM limits");
    const size_t need = fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, n_chunks);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256)
        return fail(TW_WORKSPACE, "workspace NULL, misaligned or too small (%zu < %zu bytes)", workspace_bytes, need);
    float* logits = static_cast<float*>(workspace);
    uint16_t* G = reinterpret_cast<uint16_t*>(static_cast<char*>(workspace) + (((size_t)c * vocab * 4 + 255) & ~(size_t)255));
    const bool bwd = dH || dW;

    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    rocblas_handle h;
    int rc = get_handle(&h, st);
    if (rc != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        const char* Hc = static_cast<const char*>(H) + (size_t)r0 * hidden * 2;
        // logits[n, vocab] = H_c W^T
        rc = gemm_nt(h, n, vocab, hidden, Hc, W, logits, rocblas_datatype_f32_r, 0.f);
        if (rc != TW_OK) return rc;
        loss_rows_kernel<<<dim3((unsigned)n), 256, 0, st>>>(logits, target + r0, vocab, grad_scale, loss + r0, lse + r0,
                                                             bwd ? G : nullptr);
        if (dH) {  // dH_c[n, hidden] = G[n, vocab] W[vocab, hidden]
            rc = gemm_nn(h, n, hidden, vocab, G, W, static_cast<char*>(dH) + (size_t)r0 * hidden * 2,
                         rocblas_datatype_bf16_r, 0.f);
            if (rc != TW_OK) return rc;
        }
        if (dW) {  // dW[vocab, hidden] += G^T[vocab, n] H_c[n, hidden]
            rc = gemm_tn(h, vocab, hidden, n, G, Hc, dW, rocblas_datatype_f32_r, 1.f);
            if (rc != TW_OK) return rc;
        }
    }
    HIP_TRY(hipGetLastError());
    return TW_OK;
}

const char* fpdt_tw_last_error(void) { return g_err.c_str(); }

}  // extern "C"
