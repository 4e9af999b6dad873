// Dense bf16 products of the token-wise chunked operations (Sec. 4.1, 5.4: the per-chunk QKV
// projection, the feed-forward block and the output projection of the loss are plain GEMMs over
// one chunk of tokens at a time) on v_mfma_f32_32x32x16_bf16, with the operand machinery of the
// attention kernels: operands re-laid once into 1 KiB MFMA fragments, a three-slot LDS ring
// filled by direct global -> LDS copies two stages ahead, eight waves (two per SIMD) per
// 256 x 256 output tile.
//
//   C[M,N] (+)= sum_k Aop[m,k] * Bop[n,k]          fp32 accumulation, C bf16 or fp32
//
// Every product of the library is of this form once each operand is read either as stored
// (row = row, k = column) or transposed (row = column, k = row); the pack kernel does both, pads
// rows to a multiple of 256 and k to a multiple of the stage depth with zeros, so the product kernel has no
// edge cases on its reads; its stores are bounds-checked.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <vector>

#include "mfma_tiles.h"
#include "tw_gemm.h"

namespace fpdt_tw {

using fpdt::bf16x8;
using fpdt::floatx16;
using fpdt::u32x4;

namespace {

// ---- pack -------------------------------------------------------------------------------
// X [R, C] bf16 row-major, leading dimension ld.  transposed = 0: fragment rows are rows of X,
// the contraction runs over its columns; 1: fragment rows are columns of X, the contraction
// runs over its rows.  out[rb][kt][lane][8]: lane (r = lane % 32, h = lane / 32) of fragment
// (rb, kt) holds element (row 32 rb + r, k = 16 kt + 8 h + e), e = 0..7; zero outside X.
// One workgroup: 32 fragment rows x 64 contraction indices (four fragments).
__global__ __launch_bounds__(256) void tw_pack_kernel(const uint16_t* __restrict__ X, int64_t R, int64_t C, int64_t ld,
                                                      int transposed, u32x4* __restrict__ out, int KT, int KC)
{
    __shared__ uint16_t tile[32][64 + 2];
    const int tid = threadIdx.x;
    const unsigned rb = blockIdx.x / (unsigned)KC, kc = blockIdx.x % (unsigned)KC;  // KC = chunks of 64 along k
    const int64_t row0 = (int64_t)rb * 32, k0 = (int64_t)kc * 64;
    // 256 threads x 8 consecutive elements of X = the 32 x 64 tile; 16-byte loads where the row
    // allows it (8 elements inside the matrix, 16-byte aligned), element by element at the edges
    auto load8 = [&](int64_t gr, int64_t gc0, uint16_t (&e)[8]) {
        const uint16_t* src = X + gr * ld + gc0;
        if (gr < R && gc0 + 8 <= C && (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
            const uint4 v = *reinterpret_cast<const uint4*>(src);
            e[0] = (uint16_t)v.x; e[1] = (uint16_t)(v.x >> 16); e[2] = (uint16_t)v.y; e[3] = (uint16_t)(v.y >> 16);
            e[4] = (uint16_t)v.z; e[5] = (uint16_t)(v.z >> 16); e[6] = (uint16_t)v.w; e[7] = (uint16_t)(v.w >> 16);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = (gr < R && gc0 + j < C) ? src[j] : (uint16_t)0;
        }
    };
    uint16_t e8[8];
    if (!transposed) {
        const int r = tid >> 3, k = (tid & 7) * 8;  // row r of the tile, contraction indices k .. k + 7
        load8(row0 + r, k0 + k, e8);
#pragma unroll
        for (int j = 0; j < 8; ++j) tile[r][k + j] = e8[j];
    } else {
        const int k = tid >> 2, r = (tid & 3) * 8;  // row k0 + k of X, its columns row0 + r .. + 7
        load8(k0 + k, row0 + r, e8);
#pragma unroll
        for (int j = 0; j < 8; ++j) tile[r + j][k] = e8[j];
    }
    __syncthreads();
    const int t = tid >> 6, lane = tid & 63;
    const int kt = (int)kc * 4 + t;
    if (kt < KT) {
        const int r = lane & 31, h = lane >> 5;
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = tile[r][16 * t + 8 * h + j];
        u32x4 v;
        v[0] = e[0] | ((unsigned)e[1] << 16);
        v[1] = e[2] | ((unsigned)e[3] << 16);
        v[2] = e[4] | ((unsigned)e[5] << 16);
        v[3] = e[6] | ((unsigned)e[7] << 16);
        out[((size_t)rb * KT + kt) * 64 + lane] = v;
    }
}

// ---- product ----------------------------------------------------------------------------
constexpr int NWAVE = 8, NTHREAD = NWAVE * 64;
constexpr int TILE = 256;                  // output tile: 8 row blocks x 8 column blocks of 32
#ifndef FPDT_TW_SKT
#define FPDT_TW_SKT 4
#endif
constexpr int SKT = FPDT_TW_SKT;           // k-steps of 16 per LDS stage (the packed k is a multiple of 64)
#ifndef FPDT_TW_ISSUE_LATE
#define FPDT_TW_ISSUE_LATE 0
#endif
#ifndef FPDT_TW_RING
#define FPDT_TW_RING (FPDT_TW_SKT == 2 ? 3 : 2)
#endif
constexpr int RING = FPDT_TW_RING;         // LDS slots of one stage each; RING - 1 stages are requested ahead
constexpr int OP_U4 = 8 * SKT * 64;        // the B operand of a stage (8 column blocks); A has 2 WMT row blocks

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    const unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float from_bf16(uint16_t b) { return __uint_as_float((unsigned)b << 16); }

// Af, Bf: packed operands (row blocks padded to a multiple of 8, KT a multiple of SKT).  C [M, N]
// row-major, leading dimension ldc elements.  Workgroup = 8 waves; wave (wm, wn) = (w / 4, w % 4)
// owns rows 32 WMT wm .. and columns 64 wn .. +63 of a (64 WMT) x 256 tile: WMT x 2 accumulator
// tiles.  WMT = 4 (256 x 256 tiles): every A fragment read from LDS feeds two MFMAs and every B
// fragment four, 0.75 fragments per MFMA; WMT = 2, 1 (128 and 64 rows) are for products with so
// few rows that the large tiles would leave most of the chip idle.
template <bool OUT_F32, bool ACCUM, int WMT>
__global__ __launch_bounds__(NTHREAD) void tw_gemm_kernel(const u32x4* __restrict__ Af, const u32x4* __restrict__ Bf,
                                                           int KT, void* __restrict__ Cout, int64_t ldc, int M, int N,
                                                           int tiles_n, int tiles_total)
{
    constexpr int AOP_U4 = 2 * WMT * SKT * 64;              // the A operand of a stage
    constexpr int STAGE_U4 = AOP_U4 + OP_U4;
    constexpr int NFRAG = (2 * WMT + 8) * SKT;              // fragments of a stage
    constexpr int NCOPY = NFRAG / NWAVE;                    // copied by each wave
    static_assert(NFRAG % NWAVE == 0, "every wave copies the same number of fragments");
    __shared__ u32x4 ring[RING][STAGE_U4];
    // Consecutive workgroup ids land on different XCDs (each with its own L2): give every XCD a
    // contiguous run of tiles, so that the tiles that share an operand row share an L2.
    const unsigned per_xcd = (unsigned)(tiles_total + 7) / 8;
    const unsigned id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (id >= (unsigned)tiles_total) return;  // whole workgroup, before any barrier
    // Within a run the tiles go in groups of four tile rows, row index fastest: the 32 workgroups
    // that an XCD runs at a time then cover about 4 x 8 tiles and share 4 + 8 operand slices in its
    // L2 instead of 1 + 32.
    constexpr unsigned GROUP_M = 4;
    const unsigned tiles_m = (unsigned)tiles_total / (unsigned)tiles_n;
    const unsigned grp = id / (GROUP_M * (unsigned)tiles_n), in_grp = id % (GROUP_M * (unsigned)tiles_n);
    const unsigned rows_in_grp = tiles_m - grp * GROUP_M < GROUP_M ? tiles_m - grp * GROUP_M : GROUP_M;
    const int tile_m = (int)(grp * GROUP_M + in_grp % rows_in_grp), tile_n = (int)(in_grp / rows_in_grp);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int wm = wu >> 2, wn = wu & 3;
    const int n_stages = KT / SKT;

    const u32x4* abase = Af + (size_t)tile_m * (2 * WMT) * KT * 64;
    const u32x4* bbase = Bf + (size_t)tile_n * 8 * KT * 64;
    // stage s into a slot: fragment f = wave + 8 j of the stage's 16 SKT (operand, block, k-step)
    auto issue = [&](int s, u32x4* slot) {
#pragma unroll
        for (int j = 0; j < NCOPY; ++j) {
            const int f = wu + NWAVE * j;                        // A fragments first, then B
            const bool isb = f >= 2 * WMT * SKT;
            const int g = isb ? f - 2 * WMT * SKT : f, blk = g / SKT, kt = g % SKT;
            const u32x4* src = (isb ? bbase : abase) + ((size_t)blk * KT + (size_t)s * SKT + kt) * 64;
            fpdt::frag_to_lds(src, slot + (isb ? AOP_U4 : 0) + g * 64, lane);
        }
    };

    floatx16 acc[WMT][2];
#pragma unroll
    for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    constexpr int PF = RING - 1;  // stages requested ahead
    for (int t = 0; t < PF && t < n_stages; ++t) issue(t, ring[t]);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    int slot_i = 0, pf_i = PF % RING;
    for (int s = 0; s < n_stages; ++s) {
        const u32x4* slot = ring[slot_i];
#if FPDT_TW_ISSUE_LATE == 0
        if (s + PF < n_stages) issue(s + PF, ring[pf_i]);
#endif
#pragma unroll
        for (int kt = 0; kt < SKT; ++kt) {
#if FPDT_TW_ISSUE_LATE
            // the copies go out behind the first k-step's MFMAs: right after the barrier every wave
            // of the workgroup would issue them at the same time, with no MFMA in flight
            if (kt == 1 && s + PF < n_stages) issue(s + PF, ring[pf_i]);
#endif
            bf16x8 a[WMT], b[2];
#pragma unroll
            for (int i = 0; i < WMT; ++i) a[i] = fpdt::as_bf16x8(slot[((wm * WMT + i) * SKT + kt) * 64 + lane]);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = fpdt::as_bf16x8(slot[AOP_U4 + ((wn * 2 + j) * SKT + kt) * 64 + lane]);
#pragma unroll
            for (int i = 0; i < WMT; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = fpdt::mfma32(a[i], b[j], acc[i][j]);
        }
        // stage s + 1 must have landed; the copies of the stages behind it may stay in flight
        if (s + PF < n_stages) fpdt::wait_vmem_at_most<(PF - 1) * NCOPY>();
        else fpdt::wait_vmem_at_most<0>();
        fpdt::barrier_no_fence();
        slot_i = slot_i + 1 == RING ? 0 : slot_i + 1;
        pf_i = pf_i + 1 == RING ? 0 : pf_i + 1;
    }

    // accumulator tile (i, j): lane l holds column l % 32, register r row 8 (r / 4) + 4 (l / 32) + r % 4
    const int col = lane & 31, half = lane >> 5;
#pragma unroll
    for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = tile_n * TILE + wn * 64 + j * 32 + col;
            if (n < N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = tile_m * (64 * WMT) + wm * (32 * WMT) + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (m < M) {
                        const size_t at = (size_t)m * ldc + n;
                        if (OUT_F32) {
                            float* c = static_cast<float*>(Cout);
                            c[at] = ACCUM ? c[at] + acc[i][j][r] : acc[i][j][r];
                        } else {
                            uint16_t* c = static_cast<uint16_t*>(Cout);
                            c[at] = to_bf16(ACCUM ? from_bf16(c[at]) + acc[i][j][r] : acc[i][j][r]);
                        }
                    }
                }
            }
        }
}

// ---- host side: packed-operand scratch and the per-call cache of packed weights --------------
struct Pool {
    char* base = nullptr;
    size_t cap = 0, off = 0;
    std::vector<void*> retired;  // outgrown buffers: work already enqueued may still read them
};
struct Packed {
    const void* src;
    int64_t R, C, ld;
    int transposed;
    const u32x4* frags;
    int RB, KT;
};
Pool g_pool[64];
std::vector<Packed> g_cache;  // weights packed during the current library call
std::mutex g_mu;

size_t packed_bytes(int64_t rows, int64_t k, int* RB, int* KT)
{
    *RB = (int)((rows + TILE - 1) / TILE * 8);
    *KT = (int)((k + 16 * SKT - 1) / (16 * SKT) * SKT);
    return (size_t)*RB * *KT * 1024;
}

int pool_take(Pool& p, size_t bytes, char** out)
{
    bytes = (bytes + 255) & ~(size_t)255;
    if (p.off + bytes > p.cap) {
        // grow: a new buffer; the old one stays alive (kernels in flight may read it) until exit
        size_t want = p.cap ? p.cap * 2 : (size_t)256 << 20;
        while (want < bytes) want *= 2;
        void* nb = nullptr;
        if (hipMalloc(&nb, want) != hipSuccess) {
            (void)hipGetLastError();
            return 1;
        }
        if (p.base) p.retired.push_back(p.base);
        p.base = static_cast<char*>(nb);
        p.cap = want;
        p.off = 0;
        g_cache.clear();  // cached fragments lived in the old buffer
    }
    *out = p.base + p.off;
    p.off += bytes;
    return 0;
}

int pack_operand(Pool& pool, const void* X, int64_t R, int64_t C, int64_t ld, int transposed, bool cache,
                 hipStream_t st, Packed* res)
{
    if (cache)
        for (const Packed& c : g_cache)
            if (c.src == X && c.R == R && c.C == C && c.ld == ld && c.transposed == transposed) {
                *res = c;
                return 0;
            }
    Packed p{X, R, C, ld, transposed, nullptr, 0, 0};
    const int64_t rows = transposed ? C : R, k = transposed ? R : C;
    const size_t bytes = packed_bytes(rows, k, &p.RB, &p.KT);
    char* mem = nullptr;
    if (pool_take(pool, bytes, &mem)) return 1;
    p.frags = reinterpret_cast<const u32x4*>(mem);
    const int KC = (p.KT + 3) / 4;
    if ((long long)p.RB * KC > (1ll << 30)) return 2;
    tw_pack_kernel<<<dim3((unsigned)(p.RB * KC)), 256, 0, st>>>(static_cast<const uint16_t*>(X), R, C, ld, transposed,
                                                               reinterpret_cast<u32x4*>(mem), p.KT, KC);
    if (cache) g_cache.push_back(p);
    *res = p;
    return 0;
}

}  // namespace

void begin_call()
{
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return;
    g_cache.clear();
    g_pool[dev].off = 0;  // everything enqueued earlier on the stream is ordered before what follows
}

int gemm(int a_transposed, int b_transposed, int M, int N, int K, const void* A, int64_t lda, const void* B,
         int64_t ldb, void* C, int64_t ldc, bool c_f32, bool accumulate, bool cache_b, hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1;
    Pool& pool = g_pool[dev];
    if (M <= 0 || N <= 0 || K <= 0) return 2;
    const char* base0 = pool.base;
    const size_t off0 = pool.off;
    // Aop[m,k]: A stored [M,K] (as is) or [K,M] (transposed); Bop[n,k]: B stored [N,K] or [K,N]
    Packed pa, pb;
    int rc = pack_operand(pool, B, b_transposed ? K : N, b_transposed ? N : K, ldb, b_transposed, cache_b, st, &pb);
    if (rc) return rc;
    const size_t mark = pool.off;  // what follows is scratch of this product only
    rc = pack_operand(pool, A, a_transposed ? K : M, a_transposed ? M : K, lda, a_transposed, false, st, &pa);
    if (rc) return rc;
    // 256-row tiles unless they would leave most of the chip idle: then 128 or 64 rows per tile
    const int tiles_n = (N + TILE - 1) / TILE;
    int wmt = 4;
    while (wmt > 1 && (long long)((M + 64 * wmt - 1) / (64 * wmt)) * tiles_n < 256) wmt /= 2;
    const int tiles_m = (M + 64 * wmt - 1) / (64 * wmt);
    const long long total = (long long)tiles_m * tiles_n;
    if (total > (1ll << 30)) return 2;
    const unsigned grid = (unsigned)((total + 7) / 8 * 8);
    const int KT = pa.KT;  // = pb.KT: both contract over K
#define TW_LAUNCH(F32, ACC)                                                                                                   \
    do {                                                                                                                      \
        if (wmt == 4) tw_gemm_kernel<F32, ACC, 4><<<grid, NTHREAD, 0, st>>>(pa.frags, pb.frags, KT, C, ldc, M, N, tiles_n, (int)total);      \
        else if (wmt == 2) tw_gemm_kernel<F32, ACC, 2><<<grid, NTHREAD, 0, st>>>(pa.frags, pb.frags, KT, C, ldc, M, N, tiles_n, (int)total); \
        else tw_gemm_kernel<F32, ACC, 1><<<grid, NTHREAD, 0, st>>>(pa.frags, pb.frags, KT, C, ldc, M, N, tiles_n, (int)total);               \
    } while (0)
    if (c_f32) {
        if (accumulate) TW_LAUNCH(true, true);
        else TW_LAUNCH(true, false);
    } else {
        if (accumulate) TW_LAUNCH(false, true);
        else TW_LAUNCH(false, false);
    }
#undef TW_LAUNCH
    // The next product's packs run after this launch on the same stream, so this product's scratch
    // is free again: everything it took, or everything behind a weight that stays cached.  (Not if
    // the pool was replaced by a larger one on the way: then nothing is given back until the next
    // library call.)
    if (pool.base == base0) pool.off = cache_b ? mark : off0;
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace fpdt_tw
