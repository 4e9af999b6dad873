// Token-wise chunked neighbours of the attention path (Sec. 5.4): see include/fpdt_tokenwise.h.
// The dense products are the MFMA kernels of tw_gemm.hip, the row-wise softmax / loss and the
// activations are HIP kernels of this file.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <string>

#include "../../include/fpdt_tokenwise.h"
#include "tw_gemm.h"

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
std::mutex g_mu;

// The dense products are this library's own MFMA kernels (tw_gemm.hip).  A "handle" is just the
// stream of the current call; taking it starts a call (packed weights of the previous call are
// forgotten, its scratch is reused).
struct GemmCtx { hipStream_t st; };
typedef GemmCtx* gemm_handle;
GemmCtx g_ctx;
enum { TW_C_BF16 = 0, TW_C_F32 = 1 };

int get_handle(gemm_handle* h, hipStream_t st)
{
    g_ctx.st = st;
    fpdt_tw::begin_call();
    *h = &g_ctx;
    return TW_OK;
}

int gemm_status(int rc)
{
    if (rc == 0) return TW_OK;
    if (rc == 2) return fail(TW_UNSUPPORTED, "product beyond the launch limits");
    return fail(TW_HIP, "GEMM launch or scratch allocation failed: %s", hipGetErrorString(hipGetLastError()));
}

// Row-major C[M,N] (+)= A[M,K] * B^T where B is [N,K]  ("NT": both operands K-contiguous); B is a weight.
int gemm_nt(gemm_handle h, int M, int N, int K, const void* A, const void* B, void* C, int c_type, float beta)
{
    return gemm_status(fpdt_tw::gemm(0, 0, M, N, K, A, K, B, K, C, N, c_type == TW_C_F32, beta != 0.f, true, h->st));
}
// Row-major C[M,N] (+)= A[M,K] * B[K,N]  ("NN"); B is a weight, read transposed.
int gemm_nn(gemm_handle h, int M, int N, int K, const void* A, const void* B, void* C, int c_type, float beta)
{
    return gemm_status(fpdt_tw::gemm(0, 1, M, N, K, A, K, B, N, C, N, c_type == TW_C_F32, beta != 0.f, true, h->st));
}
// Row-major C[M,N] (+)= A^T * B with A [K,M], B [K,N]  ("TN": contraction over rows, both per chunk).
int gemm_tn(gemm_handle h, int M, int N, int K, const void* A, const void* B, void* C, int c_type, float beta)
{
    return gemm_status(fpdt_tw::gemm(1, 1, M, N, K, A, M, B, N, C, N, c_type == TW_C_F32, beta != 0.f, false, h->st));
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
    // running (max, sum of exp) per thread, merged across the workgroup; rows are 16-byte
    // aligned when vocab % 4 == 0 (the base is), and then read four logits per access
    const bool vec = (vocab & 3) == 0;
    float m = -INFINITY, l = 0.f;
    if (vec) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        for (int v = tid; v < vocab / 4; v += 256) {
            const float4 a = x4[v];
            const float mn = fmaxf(fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w)), m);
            if (mn == -INFINITY) continue;  // nothing finite yet: exp(-inf - -inf) is not a number
            l = l * __expf(m - mn) + __expf(a.x - mn) + __expf(a.y - mn) + __expf(a.z - mn) + __expf(a.w - mn);
            m = mn;
        }
    } else {
        for (int v = tid; v < vocab; v += 256) {
            const float a = x[v];
            if (a > m) {
                l = l * __expf(m - a) + 1.f;
                m = a;
            } else {
                l += __expf(a - m);
            }
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
    if (vec) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        uint2* g2 = reinterpret_cast<uint2*>(g);
        for (int v = tid; v < vocab / 4; v += 256) {
            const float4 a = x4[v];
            const int d = t - 4 * v;  // 0..3 when the target is one of these four
            const unsigned p0 = to_bf16(grad_scale * (__expf(a.x - lse) - (d == 0 ? 1.f : 0.f)));
            const unsigned p1 = to_bf16(grad_scale * (__expf(a.y - lse) - (d == 1 ? 1.f : 0.f)));
            const unsigned p2 = to_bf16(grad_scale * (__expf(a.z - lse) - (d == 2 ? 1.f : 0.f)));
            const unsigned p3 = to_bf16(grad_scale * (__expf(a.w - lse) - (d == 3 ? 1.f : 0.f)));
            g2[v] = make_uint2(p0 | (p1 << 16), p2 | (p3 << 16));
        }
        return;
    }
    for (int v = tid; v < vocab; v += 256) {
        const float p = __expf(x[v] - lse) - (v == t ? 1.f : 0.f);
        g[v] = to_bf16(grad_scale * p);
    }
}

// ---- feed-forward elementwise kernels (bf16 in / out, fp32 arithmetic) ----
__device__ __forceinline__ float from_bf16(uint16_t v) { return __uint_as_float((unsigned)v << 16); }
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad(float x)
{
    return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.3989422804014327f * __expf(-0.5f * x * x);
}
__device__ __forceinline__ float sigmoid_f(float x) { return 1.f / (1.f + __expf(-x)); }

// Eight bf16 values per lane and access (16 bytes); the buffers are 256-byte aligned workspace
// tiles, and the last n % 8 elements are taken one by one.
union Bf16x8 {
    uint4 v;
    uint16_t h[8];
};

// Hh = gelu(A)  or  silu(A) * B
__global__ __launch_bounds__(256) void ffn_act_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Bm,
                                                      uint16_t* __restrict__ Hh, size_t n, int swiglu)
{
    auto one = [&](uint16_t a16, uint16_t b16) {
        const float a = from_bf16(a16);
        return to_bf16(swiglu ? a * sigmoid_f(a) * from_bf16(b16) : gelu_f(a));
    };
    const size_t n8 = n / 8;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        Bf16x8 a, b, o;
        a.v = reinterpret_cast<const uint4*>(A)[i];
        b.v = swiglu ? reinterpret_cast<const uint4*>(Bm)[i] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) o.h[e] = one(a.h[e], b.h[e]);
        reinterpret_cast<uint4*>(Hh)[i] = o.v;
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n8 * 8) {
        const size_t i = n8 * 8 + threadIdx.x;
        Hh[i] = one(A[i], swiglu ? Bm[i] : (uint16_t)0);
    }
}
// dA = dHh * act'(A) (* B);  SWIGLU also dB = dHh * silu(A).  dA overwrites A, dB overwrites B.
__global__ __launch_bounds__(256) void ffn_act_grad_kernel(uint16_t* __restrict__ A, uint16_t* __restrict__ Bm,
                                                           const uint16_t* __restrict__ dHh, size_t n, int swiglu)
{
    auto one = [&](uint16_t& a16, uint16_t& b16, uint16_t g16) {
        const float a = from_bf16(a16), g = from_bf16(g16);
        if (swiglu) {
            const float b = from_bf16(b16), sg = sigmoid_f(a);
            a16 = to_bf16(g * b * sg * (1.f + a * (1.f - sg)));
            b16 = to_bf16(g * a * sg);
        } else {
            a16 = to_bf16(g * gelu_grad(a));
        }
    };
    const size_t n8 = n / 8;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        Bf16x8 a, b, g;
        a.v = reinterpret_cast<const uint4*>(A)[i];
        g.v = reinterpret_cast<const uint4*>(dHh)[i];
        b.v = swiglu ? reinterpret_cast<const uint4*>(Bm)[i] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) one(a.h[e], b.h[e], g.h[e]);
        reinterpret_cast<uint4*>(A)[i] = a.v;
        if (swiglu) reinterpret_cast<uint4*>(Bm)[i] = b.v;
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n8 * 8) {
        const size_t i = n8 * 8 + threadIdx.x;
        uint16_t a = A[i], b = swiglu ? Bm[i] : (uint16_t)0;
        one(a, b, dHh[i]);
        A[i] = a;
        if (swiglu) Bm[i] = b;
    }
}
unsigned ew_blocks(size_t n)
{
    size_t b = (n / 8 + 255) / 256;
    return (unsigned)(b > 8192 ? 8192 : (b ? b : 1));  // grid-stride loops take the rest
}
size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_chunking(int64_t rows, int n_chunks)
{
    if (rows <= 0) return fail(TW_INVALID, "rows must be positive");
    if (n_chunks <= 0 || n_chunks > rows) return fail(TW_INVALID, "n_chunks=%d must be in [1, rows]", n_chunks);
    if ((rows + n_chunks - 1) / n_chunks > (int64_t)1 << 24) return fail(TW_UNSUPPORTED, "chunk beyond the 32-bit GEMM limits");
    return TW_OK;
}

}  // namespace

extern "C" {

int fpdt_tw_linear_fwd(const void* X, const void* W, void* Y, int64_t rows, int n_in, int n_out, int n_chunks,
                       void* stream)
{
    g_err.clear();
    if (!X || !W || !Y) return fail(TW_INVALID, "NULL tensor pointer");
    if (n_in <= 0 || n_out <= 0) return fail(TW_INVALID, "n_in and n_out must be positive");
    int rc = check_chunking(rows, n_chunks);
    if (rc != TW_OK) return rc;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    gemm_handle h;
    if ((rc = get_handle(&h, st)) != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        rc = gemm_nt(h, n, n_out, n_in, static_cast<const char*>(X) + (size_t)r0 * n_in * 2, W,
                     static_cast<char*>(Y) + (size_t)r0 * n_out * 2, TW_C_BF16, 0.f);
        if (rc != TW_OK) return rc;
    }
    return TW_OK;
}

int fpdt_tw_linear_bwd(const void* X, const void* W, const void* dY, void* dX, float* dW, int64_t rows, int n_in,
                       int n_out, int n_chunks, void* stream)
{
    g_err.clear();
    if (!X || !W || !dY) return fail(TW_INVALID, "NULL tensor pointer");
    if (n_in <= 0 || n_out <= 0) return fail(TW_INVALID, "n_in and n_out must be positive");
    int rc = check_chunking(rows, n_chunks);
    if (rc != TW_OK) return rc;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    gemm_handle h;
    if ((rc = get_handle(&h, st)) != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        const char* dYc = static_cast<const char*>(dY) + (size_t)r0 * n_out * 2;
        if (dX) {  // dX_c[n, n_in] = dY_c[n, n_out] W[n_out, n_in]
            rc = gemm_nn(h, n, n_in, n_out, dYc, W, static_cast<char*>(dX) + (size_t)r0 * n_in * 2, TW_C_BF16, 0.f);
            if (rc != TW_OK) return rc;
        }
        if (dW) {  // dW[n_out, n_in] += dY_c^T X_c
            rc = gemm_tn(h, n_out, n_in, n, dYc, static_cast<const char*>(X) + (size_t)r0 * n_in * 2, dW, TW_C_F32, 1.f);
            if (rc != TW_OK) return rc;
        }
    }
    return TW_OK;
}

size_t fpdt_tw_ffn_workspace_bytes(int64_t rows, int n_model, int n_ffn, int act, int n_chunks, int is_bwd)
{
    if (rows <= 0 || n_model <= 0 || n_ffn <= 0 || n_chunks <= 0 || n_chunks > rows) return 0;
    if (act != FPDT_TW_GELU && act != FPDT_TW_SWIGLU) return 0;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    const size_t t = al256((size_t)c * n_ffn * 2);  // one [chunk, n_ffn] bf16 intermediate
    // forward: A, (B), Hh;  backward: A, (B), Hh, dHh
    return t * ((act == FPDT_TW_SWIGLU ? 3 : 2) + (is_bwd ? 1 : 0));
}

static int ffn_common(const void* X, const void* W1, const void* W3, const void* W2, int64_t rows, int n_model,
                      int n_ffn, int act, int n_chunks, void* workspace, size_t workspace_bytes, int is_bwd)
{
    g_err.clear();
    if (!X || !W1 || !W2) return fail(TW_INVALID, "NULL tensor pointer");
    if (act != FPDT_TW_GELU && act != FPDT_TW_SWIGLU) return fail(TW_INVALID, "unknown activation %d", act);
    if (act == FPDT_TW_SWIGLU && !W3) return fail(TW_INVALID, "SWIGLU needs W3");
    if (n_model <= 0 || n_ffn <= 0) return fail(TW_INVALID, "n_model and n_ffn must be positive");
    int rc = check_chunking(rows, n_chunks);
    if (rc != TW_OK) return rc;
    const size_t need = fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, act, n_chunks, is_bwd);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256)
        return fail(TW_WORKSPACE, "workspace NULL, misaligned or too small (%zu < %zu bytes)", workspace_bytes, need);
    return TW_OK;
}

int fpdt_tw_ffn_fwd(const void* X, const void* W1, const void* W3, const void* W2, void* Y, int64_t rows,
                    int n_model, int n_ffn, int act, int n_chunks, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    int rc = ffn_common(X, W1, W3, W2, rows, n_model, n_ffn, act, n_chunks, workspace, workspace_bytes, 0);
    if (rc != TW_OK) return rc;
    if (!Y) return fail(TW_INVALID, "NULL tensor pointer");
    const bool sw = act == FPDT_TW_SWIGLU;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    const size_t t = al256((size_t)c * n_ffn * 2);
    char* ws = static_cast<char*>(workspace);
    uint16_t* A = reinterpret_cast<uint16_t*>(ws);
    uint16_t* Bm = sw ? reinterpret_cast<uint16_t*>(ws + t) : nullptr;
    uint16_t* Hh = reinterpret_cast<uint16_t*>(ws + (sw ? 2 : 1) * t);
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    gemm_handle h;
    if ((rc = get_handle(&h, st)) != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        const char* Xc = static_cast<const char*>(X) + (size_t)r0 * n_model * 2;
        if ((rc = gemm_nt(h, n, n_ffn, n_model, Xc, W1, A, TW_C_BF16, 0.f)) != TW_OK) return rc;
        if (sw && (rc = gemm_nt(h, n, n_ffn, n_model, Xc, W3, Bm, TW_C_BF16, 0.f)) != TW_OK) return rc;
        const size_t ne = (size_t)n * n_ffn;
        ffn_act_kernel<<<dim3(ew_blocks(ne)), 256, 0, st>>>(A, Bm, Hh, ne, sw);
        if ((rc = gemm_nt(h, n, n_model, n_ffn, Hh, W2, static_cast<char*>(Y) + (size_t)r0 * n_model * 2,
                          TW_C_BF16, 0.f)) != TW_OK) return rc;
    }
    HIP_TRY(hipGetLastError());
    return TW_OK;
}

int fpdt_tw_ffn_bwd(const void* X, const void* W1, const void* W3, const void* W2, const void* dY, void* dX,
                    float* dW1, float* dW3, float* dW2, int64_t rows, int n_model, int n_ffn, int act, int n_chunks,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = ffn_common(X, W1, W3, W2, rows, n_model, n_ffn, act, n_chunks, workspace, workspace_bytes, 1);
    if (rc != TW_OK) return rc;
    if (!dY || !dX) return fail(TW_INVALID, "NULL tensor pointer");
    const bool sw = act == FPDT_TW_SWIGLU;
    const int64_t c = (rows + n_chunks - 1) / n_chunks;
    const size_t t = al256((size_t)c * n_ffn * 2);
    char* ws = static_cast<char*>(workspace);
    uint16_t* A = reinterpret_cast<uint16_t*>(ws);
    uint16_t* Bm = sw ? reinterpret_cast<uint16_t*>(ws + t) : nullptr;
    uint16_t* Hh = reinterpret_cast<uint16_t*>(ws + (sw ? 2 : 1) * t);
    uint16_t* dHh = reinterpret_cast<uint16_t*>(ws + (sw ? 3 : 2) * t);
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    gemm_handle h;
    if ((rc = get_handle(&h, st)) != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        const char* Xc = static_cast<const char*>(X) + (size_t)r0 * n_model * 2;
        const char* dYc = static_cast<const char*>(dY) + (size_t)r0 * n_model * 2;
        char* dXc = static_cast<char*>(dX) + (size_t)r0 * n_model * 2;
        const size_t ne = (size_t)n * n_ffn;
        // recompute the chunk's pre-activations and hidden activations
        if ((rc = gemm_nt(h, n, n_ffn, n_model, Xc, W1, A, TW_C_BF16, 0.f)) != TW_OK) return rc;
        if (sw && (rc = gemm_nt(h, n, n_ffn, n_model, Xc, W3, Bm, TW_C_BF16, 0.f)) != TW_OK) return rc;
        if (dW2) {
            ffn_act_kernel<<<dim3(ew_blocks(ne)), 256, 0, st>>>(A, Bm, Hh, ne, sw);
            // dW2[n_model, n_ffn] += dY_c^T Hh
            if ((rc = gemm_tn(h, n_model, n_ffn, n, dYc, Hh, dW2, TW_C_F32, 1.f)) != TW_OK) return rc;
        }
        // dHh[n, n_ffn] = dY_c[n, n_model] W2[n_model, n_ffn]
        if ((rc = gemm_nn(h, n, n_ffn, n_model, dYc, W2, dHh, TW_C_BF16, 0.f)) != TW_OK) return rc;
        ffn_act_grad_kernel<<<dim3(ew_blocks(ne)), 256, 0, st>>>(A, Bm, dHh, ne, sw);  // A <- dA, B <- dB
        // dX_c = dA W1 (+ dB W3)
        if ((rc = gemm_nn(h, n, n_model, n_ffn, A, W1, dXc, TW_C_BF16, 0.f)) != TW_OK) return rc;
        if (sw && (rc = gemm_nn(h, n, n_model, n_ffn, Bm, W3, dXc, TW_C_BF16, 1.f)) != TW_OK) return rc;
        if (dW1 && (rc = gemm_tn(h, n_ffn, n_model, n, A, Xc, dW1, TW_C_F32, 1.f)) != TW_OK) return rc;
        if (sw && dW3 && (rc = gemm_tn(h, n_ffn, n_model, n, Bm, Xc, dW3, TW_C_F32, 1.f)) != TW_OK) return rc;
    }
    HIP_TRY(hipGetLastError());
    return TW_OK;
}

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
    gemm_handle h;
    int rc = get_handle(&h, st);
    if (rc != TW_OK) return rc;
    for (int64_t r0 = 0; r0 < rows; r0 += c) {
        const int n = (int)(rows - r0 < c ? rows - r0 : c);
        const char* Hc = static_cast<const char*>(H) + (size_t)r0 * hidden * 2;
        // logits[n, vocab] = H_c W^T
        rc = gemm_nt(h, n, vocab, hidden, Hc, W, logits, TW_C_F32, 0.f);
        if (rc != TW_OK) return rc;
        loss_rows_kernel<<<dim3((unsigned)n), 256, 0, st>>>(logits, target + r0, vocab, grad_scale, loss + r0, lse + r0,
                                                             bwd ? G : nullptr);
        if (dH) {  // dH_c[n, hidden] = G[n, vocab] W[vocab, hidden]
            rc = gemm_nn(h, n, hidden, vocab, G, W, static_cast<char*>(dH) + (size_t)r0 * hidden * 2,
                         TW_C_BF16, 0.f);
            if (rc != TW_OK) return rc;
        }
        if (dW) {  // dW[vocab, hidden] += G^T[vocab, n] H_c[n, hidden]
            rc = gemm_tn(h, vocab, hidden, n, G, Hc, dW, TW_C_F32, 1.f);
            if (rc != TW_OK) return rc;
        }
    }
    HIP_TRY(hipGetLastError());
    return TW_OK;
}

const char* fpdt_tw_last_error(void) { return g_err.c_str(); }

}  // extern "C"
