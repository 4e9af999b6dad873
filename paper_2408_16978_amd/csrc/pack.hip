// Re-layout of [rows, H, D] bf16 tensors into MFMA fragment order (see fpdt_internal.h).
// HBM-bound streaming kernel: each workgroup stages one 32-row x D tile of one head in
// LDS and writes it back as NAT and/or TR fragments, 16 bytes per lane, fully coalesced.
#include "fpdt_internal.h"
#include "mfma_tiles.h"

namespace fpdt {

template <int D>
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ X, int H,
                                                   uint4* __restrict__ nat, uint4* __restrict__ tr,
                                                   int64_t head_stride_blocks)
{
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int LD = DP + 2;  // padded row (in bf16) to spread LDS banks on column reads
    __shared__ uint16_t tile[32 * LD];
    const int64_t rb = blockIdx.x;
    const int h = blockIdx.y;
    const int tid = threadIdx.x;
    // load 32 rows x D (8 bf16 = 16 B per thread per step)
    constexpr int VEC_PER_ROW = D / 8;
    for (int i = tid; i < 32 * VEC_PER_ROW; i += 256) {
        const int r = i / VEC_PER_ROW, c = (i % VEC_PER_ROW) * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(X + ((size_t)(rb * 32 + r) * H + h) * D + c);
        const uint16_t* e = reinterpret_cast<const uint16_t*>(&v);
#pragma unroll
        for (int k = 0; k < 8; ++k) tile[r * LD + c + k] = e[k];
    }
    if (DP != D) {
        for (int i = tid; i < 32 * (DP - D); i += 256) {
            const int r = i / (DP - D), c = D + i % (DP - D);
            tile[r * LD + c] = 0;
        }
    }
    __syncthreads();
    const size_t blk = (size_t)h * head_stride_blocks + rb;
    if (nat) {
        uint4* out = nat + blk * (DT * 64);
        for (int i = tid; i < DT * 64; i += 256) {
            const int t = i >> 6, lane = i & 63;
            const int r = lane & 31, hh = lane >> 5;
            uint16_t e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e[k] = tile[r * LD + 16 * t + 8 * hh + k];
            out[i] = *reinterpret_cast<const uint4*>(e);
        }
    }
    if (tr) {
        uint4* out = tr + blk * (2 * DB * 64);
        for (int i = tid; i < 2 * DB * 64; i += 256) {
            const int lane = i & 63, db = (i >> 6) % DB, s = (i >> 6) / DB;
            const int c = lane & 31, hh = lane >> 5;
            uint16_t e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                e[k] = tile[(8 * (2 * s + (k >> 2)) + 4 * hh + (k & 3)) * LD + 32 * db + c];
            out[i] = *reinterpret_cast<const uint4*>(e);
        }
    }
}

void launch_pack(const void* X, int64_t rows, int H, int D, void* nat, void* tr,
                 int64_t head_stride_blocks, hipStream_t st)
{
    if (rows <= 0) return;
    dim3 grid((unsigned)(rows / 32), (unsigned)H);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint4* n = static_cast<uint4*>(nat);
    uint4* t = static_cast<uint4*>(tr);
    if (D == 128) pack_kernel<128><<<grid, 256, 0, st>>>(x, H, n, t, head_stride_blocks);
    else if (D == 80) pack_kernel<80><<<grid, 256, 0, st>>>(x, H, n, t, head_stride_blocks);
    else pack_kernel<64><<<grid, 256, 0, st>>>(x, H, n, t, head_stride_blocks);
}

}  // namespace fpdt
