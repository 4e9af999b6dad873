// Calibration loops for the roofline discussion of the attention kernels (not on the hot path):
// what one MI355X sustains on v_mfma_f32_32x32x16_bf16 with RANDOM bf16 operands (the chip's
// clock under load depends on the data), alone and in the company the attention kernels keep:
// the softmax's vector instructions issued between the MFMAs, and A operands that are freshly
// read from LDS (one 1 KiB fragment per MFMA, or one per two MFMAs).  Every loop is pure
// register / LDS work of a fixed trip count; nothing is read from or written to global memory
// inside it.
#include "fpdt_internal.h"
#include "mfma_tiles.h"

namespace fpdt {

namespace {

#define CAL_MFMA(d, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b))

// Four vector instructions per MFMA, the per-element mix of the forward's online softmax:
// multiply-add, exp2, add, and alternately a packed bf16 conversion or a three-way maximum.
__device__ __forceinline__ void softmax_mix4(float (&x)[8], unsigned& pk, float m, float ad, int odd)
{
    if (!odd) {
        asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[0]) : "v"(m), "v"(ad));
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[1]));
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[2]) : "v"(ad));
        asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(x[1]), "v"(x[4]));
    } else {
        asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[3]) : "v"(m), "v"(ad));
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[4]));
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[5]) : "v"(ad));
        asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x[7]) : "v"(x[0]), "v"(x[3]));
    }
}

// LDS_MODE: 0 register operands, 1 one LDS fragment per MFMA, 2 one LDS fragment per two MFMAs.
template <int LDS_MODE, bool VALU, int NT>
__global__ __launch_bounds__(NT) void calibrate_kernel(float* out, const u32x4* in, int iters)
{
    constexpr int NFRAG = 32;  // 32 KiB of operand fragments, re-read in a rotating order
    __shared__ u32x4 frag[LDS_MODE ? NFRAG * 64 : 64];
    const int lane = threadIdx.x & 63;
    if (LDS_MODE)
        for (int i = threadIdx.x; i < NFRAG * 64; i += NT) frag[i] = in[i & 127] ^ (u32x4){(unsigned)(i >> 7) << 16, 0u, (unsigned)(i >> 7), 0u};
    __syncthreads();
    const bf16x8 b0 = as_bf16x8(in[64 + lane]), b1 = as_bf16x8(in[lane ^ 17]);
    bf16x8 a = as_bf16x8(in[lane]);
    floatx16 c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[t][r] = 0.f;
    float x[8];
    unsigned pk = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) x[r] = __builtin_bit_cast(float, in[lane][r & 3]) * 1e-3f + 0.01f * r;
    const float m = 0.999f, ad = 0.001f;
    bf16x8 fr[6];
    int pos = (threadIdx.x >> 6) * 5;  // waves start at different fragments
    auto next = [&]() { const bf16x8 v = as_bf16x8(frag[(pos & (NFRAG - 1)) * 64 + lane]); ++pos; return v; };
    if (LDS_MODE) {
#pragma unroll
        for (int u = 0; u < 4; ++u) fr[u] = next();
    }
    for (int i = 0; i < iters; ++i) {
        // 24 MFMAs per trip (a multiple of the six-deep fragment ring and of the four accumulators)
#pragma unroll
        for (int u = 0; u < 24; ++u) {
            if (LDS_MODE == 0) {
                CAL_MFMA(c[u & 3], a, (u & 1) ? b1 : b0);
            } else if (LDS_MODE == 1) {
                CAL_MFMA(c[u & 3], fr[u % 6], b0);
                fr[(u + 4) % 6] = next();
            } else {
                CAL_MFMA(c[u & 3], fr[(u / 2) % 6], (u & 1) ? b1 : b0);
                if (u & 1) fr[(u / 2 + 4) % 6] = next();
            }
            if (VALU) softmax_mix4(x, pk, m, ad, u & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float s = __builtin_bit_cast(float, pk);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[t][r];
#pragma unroll
    for (int r = 0; r < 8; ++r) s += x[r];
    if (LDS_MODE) {
#pragma unroll
        for (int u = 0; u < 6; ++u) s += (float)fr[u][0];
    }
    out[(size_t)blockIdx.x * NT + threadIdx.x] = s;
}

template <int LDS_MODE, bool VALU, int NT>
void launch(float* out, const u32x4* in, int iters, int blocks, hipStream_t st)
{
    calibrate_kernel<LDS_MODE, VALU, NT><<<blocks, NT, 0, st>>>(out, in, iters);
}

__global__ void calibrate_fill_kernel(unsigned* in, int n)
{
    // bf16 pairs with random mantissas and signs, exponents of 0.5 .. 2: magnitudes of order one
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    unsigned s = 12345u + 2654435761u * (unsigned)i;
    s = s * 1664525u + 1013904223u;
    s ^= s >> 15;
    s = s * 1664525u + 1013904223u;
    const unsigned lo = 0x3f00u + (s & 0x00ffu) + ((s >> 8) & 0x8000u);
    const unsigned hi = 0x3f00u + ((s >> 8) & 0x00ffu) + ((s >> 1) & 0x8000u);
    in[i] = lo | (hi << 16);
}

}  // namespace

void launch_calibrate_fill(void* in, hipStream_t st)
{
    calibrate_fill_kernel<<<2, 256, 0, st>>>(static_cast<unsigned*>(in), 512);
}

// out: blocks * 512 floats of scratch output; in: 128 u32x4 of random bf16 pairs.
// One workgroup per launched block, 256 threads (one wave per SIMD) or 512 (two).
int launch_calibrate(int kind, float* out, const void* in, int iters, int blocks, hipStream_t st)
{
    const u32x4* p = static_cast<const u32x4*>(in);
    switch (kind) {
    case 0: launch<0, false, 512>(out, p, iters, blocks, st); return 2;
    case 1: launch<0, false, 256>(out, p, iters, blocks, st); return 1;
    case 2: launch<0, true, 512>(out, p, iters, blocks, st); return 2;
    case 3: launch<0, true, 256>(out, p, iters, blocks, st); return 1;
    case 4: launch<1, false, 512>(out, p, iters, blocks, st); return 2;
    case 5: launch<2, false, 256>(out, p, iters, blocks, st); return 1;
    case 6: launch<1, true, 512>(out, p, iters, blocks, st); return 2;
    case 7: launch<2, true, 256>(out, p, iters, blocks, st); return 1;
    default: return 0;
    }
}

}  // namespace fpdt
