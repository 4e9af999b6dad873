// fp32 accuracy path, partial-result merge and fill kernels.
//
// The fp32 kernels run the same chunk-pair schedule as the bf16 path (Sec. 4.1 / 4.2) with
// plain FMA arithmetic: one wavefront per row, lanes split the keys (or queries) of a block
// of 64 for the dot products and split the channels for the accumulations.  They exist for
// accuracy (fp32 tensors, 1e-4 class agreement with the definition), not for speed.
#include "fpdt_internal.h"

namespace fpdt {

namespace {

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
__device__ __forceinline__ float dotD(const float* __restrict__ a, const float* __restrict__ b, int D)
{
    float acc = 0.f;
    for (int d = 0; d < D; d += 4) {
        const float4 x = *reinterpret_cast<const float4*>(a + d);
        const float4 y = *reinterpret_cast<const float4*>(b + d);
        acc = fmaf(x.x, y.x, acc);
        acc = fmaf(x.y, y.y, acc);
        acc = fmaf(x.z, y.z, acc);
        acc = fmaf(x.w, y.w, acc);
    }
    return acc;
}

// One wave per (query row, head).  Folds keys [0, n_k) of the pair into the row's carried
// (max, sum, un-normalised output).
__global__ __launch_bounds__(256) void f32_fwd_pair_kernel(F32FwdArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= a.n_q * a.Hq) return;  // wave-uniform
    const int64_t row = pair / a.Hq;
    const int head = (int)(pair % a.Hq);
    const int kvh = head / (a.Hq / a.Hkv);
    const int D = a.D;
    const float* q = a.Q + ((size_t)row * a.Hq + head) * D;
    const int d0 = lane, d1 = lane + 64;

    float m, l, acc0, acc1;
    float* sacc = a.st_acc + ((size_t)row * a.Hq + head) * D;
    float* sml = a.st_ml + ((size_t)row * a.Hq + head) * 2;
    if (a.flags & SWEEP_INIT) {
        m = -INFINITY; l = 0.f; acc0 = acc1 = 0.f;
    } else {
        m = sml[0]; l = sml[1];
        acc0 = d0 < D ? sacc[d0] : 0.f;
        acc1 = d1 < D ? sacc[d1] : 0.f;
    }
    int64_t n_valid = a.q_pos0 + row - a.k_pos0 + 1;  // keys at positions <= the query's
    if (n_valid > a.n_k) n_valid = a.n_k;
    for (int64_t j0 = 0; j0 < n_valid; j0 += 64) {
        const int64_t j = j0 + lane;
        const bool valid = j < n_valid;
        const float s = valid ? a.scale * dotD(q, a.K + ((size_t)j * a.Hkv + kvh) * D, D) : -INFINITY;
        const float m_new = fmaxf(m, wave_max(s));
        const float alpha = expf(m - m_new);
        const float p = valid ? expf(s - m_new) : 0.f;
        l = l * alpha + wave_sum(p);
        acc0 *= alpha; acc1 *= alpha;
        const int cnt = (int)((n_valid - j0) < 64 ? (n_valid - j0) : 64);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const float* v = a.V + ((size_t)(j0 + jj) * a.Hkv + kvh) * D;
            if (d0 < D) acc0 = fmaf(pj, v[d0], acc0);
            if (d1 < D) acc1 = fmaf(pj, v[d1], acc1);
        }
        m = m_new;
    }
    if (a.flags & SWEEP_FINAL) {
        float* o = a.O + ((size_t)row * a.Hq + head) * D;
        const float inv = 1.f / l;
        if (d0 < D) o[d0] = acc0 * inv;
        if (d1 < D) o[d1] = acc1 * inv;
        if (lane == 0) a.LSE[(size_t)head * a.lse_stride + row] = m + logf(l);
    } else {
        if (d0 < D) sacc[d0] = acc0;
        if (d1 < D) sacc[d1] = acc1;
        if (lane == 0) { sml[0] = m; sml[1] = l; }
    }
}

// dQ share of one chunk pair: one wave per (query row, head).
__global__ __launch_bounds__(256) void f32_bwd_dq_kernel(F32BwdArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= a.n_q * a.Hq) return;
    const int64_t row = pair / a.Hq;
    const int head = (int)(pair % a.Hq);
    const int kvh = head / (a.Hq / a.Hkv);
    const int D = a.D;
    const float* q = a.Q + ((size_t)row * a.Hq + head) * D;
    const float* go = a.dO + ((size_t)row * a.Hq + head) * D;
    const float lse = a.LSE[(size_t)head * a.row_stat_stride + row];
    const float delta = a.Delta[(size_t)head * a.row_stat_stride + row];
    const int d0 = lane, d1 = lane + 64;
    float g0 = 0.f, g1 = 0.f;
    int64_t n_valid = a.q_pos0 + row - a.k_pos0 + 1;
    if (n_valid > a.n_k) n_valid = a.n_k;
    for (int64_t j0 = 0; j0 < n_valid; j0 += 64) {
        const int64_t j = j0 + lane;
        float ds = 0.f;
        if (j < n_valid) {
            const float* k = a.K + ((size_t)j * a.Hkv + kvh) * D;
            const float* v = a.V + ((size_t)j * a.Hkv + kvh) * D;
            const float p = expf(a.scale * dotD(q, k, D) - lse);
            ds = p * (dotD(go, v, D) - delta);
        }
        const int cnt = (int)((n_valid - j0) < 64 ? (n_valid - j0) : 64);
        for (int jj = 0; jj < cnt; ++jj) {
            const float dj = __shfl(ds, jj, 64);
            const float* k = a.K + ((size_t)(j0 + jj) * a.Hkv + kvh) * D;
            if (d0 < D) g0 = fmaf(dj, k[d0], g0);
            if (d1 < D) g1 = fmaf(dj, k[d1], g1);
        }
    }
    float* out = a.dQ + ((size_t)row * a.Hq + head) * D;
    if (d0 < D) out[d0] += a.scale * g0;
    if (d1 < D) out[d1] += a.scale * g1;
}

// dK, dV share of one chunk pair: one wave per (key row, KV head), summing over the group's
// query heads and the query rows at or after the key.
__global__ __launch_bounds__(256) void f32_bwd_dkdv_kernel(F32BwdArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= a.n_k * a.Hkv) return;
    const int64_t krow = pair / a.Hkv;
    const int kvh = (int)(pair % a.Hkv);
    const int g = a.Hq / a.Hkv;
    const int D = a.D;
    const float* k = a.K + ((size_t)krow * a.Hkv + kvh) * D;
    const float* v = a.V + ((size_t)krow * a.Hkv + kvh) * D;
    const int d0 = lane, d1 = lane + 64;
    float gk0 = 0.f, gk1 = 0.f, gv0 = 0.f, gv1 = 0.f;
    int64_t i_first = a.k_pos0 + krow - a.q_pos0;  // first query row that attends this key
    if (i_first < 0) i_first = 0;
    for (int head = kvh * g; head < (kvh + 1) * g; ++head) {
        for (int64_t i0 = i_first; i0 < a.n_q; i0 += 64) {
            const int64_t i = i0 + lane;
            float p = 0.f, ds = 0.f;
            if (i < a.n_q) {
                const float* q = a.Q + ((size_t)i * a.Hq + head) * D;
                const float* go = a.dO + ((size_t)i * a.Hq + head) * D;
                p = expf(a.scale * dotD(q, k, D) - a.LSE[(size_t)head * a.row_stat_stride + i]);
                ds = p * (dotD(go, v, D) - a.Delta[(size_t)head * a.row_stat_stride + i]);
            }
            const int cnt = (int)((a.n_q - i0) < 64 ? (a.n_q - i0) : 64);
            for (int ii = 0; ii < cnt; ++ii) {
                const float pi = __shfl(p, ii, 64), di = __shfl(ds, ii, 64);
                const float* q = a.Q + ((size_t)(i0 + ii) * a.Hq + head) * D;
                const float* go = a.dO + ((size_t)(i0 + ii) * a.Hq + head) * D;
                if (d0 < D) { gk0 = fmaf(di, q[d0], gk0); gv0 = fmaf(pi, go[d0], gv0); }
                if (d1 < D) { gk1 = fmaf(di, q[d1], gk1); gv1 = fmaf(pi, go[d1], gv1); }
            }
        }
    }
    float* ok = a.dK + ((size_t)krow * a.Hkv + kvh) * D;
    float* ov = a.dV + ((size_t)krow * a.Hkv + kvh) * D;
    if (d0 < D) { ok[d0] += a.scale * gk0; ov[d0] += gv0; }
    if (d1 < D) { ok[d1] += a.scale * gk1; ov[d1] += gv1; }
}

__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t* p) { return __uint_as_float(((unsigned)*p) << 16); }
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, float v)
{
    const __bf16 b = (__bf16)v;  // round to nearest even
    *p = __builtin_bit_cast(uint16_t, b);
}

// 16 lanes per (row, head).
template <typename T>
__global__ __launch_bounds__(256) void merge_kernel(const T* Oa, const float* La, const T* Ob,
                                                    const float* Lb, T* Oo, float* Lo, int64_t rows,
                                                    int Hq, int D)
{
    const int64_t pair = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int sub = threadIdx.x & 15;
    if (pair >= rows * Hq) return;
    const int64_t row = pair / Hq;
    const int h = (int)(pair % Hq);
    const float la = La[(size_t)h * rows + row], lb = Lb[(size_t)h * rows + row];
    const float mx = fmaxf(la, lb);
    float lse = -INFINITY, wa = 0.f, wb = 0.f;
    if (mx > -INFINITY) {
        lse = mx + logf(expf(la - mx) + expf(lb - mx));
        wa = expf(la - lse);
        wb = expf(lb - lse);
    }
    for (int d = sub; d < D; d += 16) {
        const size_t o = (size_t)pair * D + d;
        const float xa = wa > 0.f ? load_elem(Oa + o) : 0.f;
        const float xb = wb > 0.f ? load_elem(Ob + o) : 0.f;
        store_elem(Oo + o, wa * xa + wb * xb);
    }
    if (sub == 0) Lo[(size_t)h * rows + row] = lse;
}

__global__ __launch_bounds__(256) void fill_kernel(uint4* p, size_t n16, unsigned char* tail, int ntail, unsigned word)
{
    const size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t step = (size_t)gridDim.x * 256;
    for (size_t i = i0; i < n16; i += step) p[i] = make_uint4(word, word, word, word);
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = (unsigned char)word;
}

}  // namespace

void launch_f32_fwd_pair(const F32FwdArgs& a, hipStream_t st)
{
    const int64_t pairs = a.n_q * a.Hq;
    f32_fwd_pair_kernel<<<dim3((unsigned)((pairs + 3) / 4)), 256, 0, st>>>(a);
}

void launch_f32_bwd_pair(const F32BwdArgs& a, hipStream_t st)
{
    const int64_t qp = a.n_q * a.Hq, kp = a.n_k * a.Hkv;
    f32_bwd_dq_kernel<<<dim3((unsigned)((qp + 3) / 4)), 256, 0, st>>>(a);
    f32_bwd_dkdv_kernel<<<dim3((unsigned)((kp + 3) / 4)), 256, 0, st>>>(a);
}

void launch_merge(const void* Oa, const float* La, const void* Ob, const float* Lb, void* Oo,
                  float* Lo, int64_t rows, int Hq, int D, int is_bf16, hipStream_t st)
{
    const int64_t pairs = rows * Hq;
    dim3 grid((unsigned)((pairs + 15) / 16));
    if (is_bf16)
        merge_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)Oa, La, (const uint16_t*)Ob, Lb,
                                                     (uint16_t*)Oo, Lo, rows, Hq, D);
    else
        merge_kernel<float><<<grid, 256, 0, st>>>((const float*)Oa, La, (const float*)Ob, Lb,
                                                  (float*)Oo, Lo, rows, Hq, D);
}

void launch_zero(void* p, size_t bytes, hipStream_t st) { launch_fill_bytes(p, bytes, 0x00, st); }

void launch_fill_bytes(void* p, size_t bytes, unsigned char byte, hipStream_t st)
{
    if (bytes == 0) return;
    const unsigned word = 0x01010101u * byte;
    const size_t n16 = bytes / 16;
    const int ntail = (int)(bytes % 16);
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks == 0) blocks = 1;
    fill_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>((uint4*)p, n16, (unsigned char*)p + n16 * 16, ntail, word);
}

}  // namespace fpdt
