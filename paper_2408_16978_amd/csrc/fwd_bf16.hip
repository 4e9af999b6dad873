// Forward chunk sweep on bf16 MFMA (Sec. 4.1: query chunk against key/value chunks with
// online-softmax accumulation; causal mask only where the key range reaches the queries).
//
// Formulation: the score tile is computed transposed, S^T = K Q^T (keys are MFMA rows,
// queries are MFMA columns).  In the 32x32 accumulator layout a lane then owns ONE query
// (column lane%32) and 16 keys, so the running max / sum of a query are lane-local up to a
// single exchange between lanes l and l+32, and the exponentiated tile -- still in
// registers -- is directly the B operand of O^T += V^T P^T.  K arrives as NAT fragments,
// V as TR fragments (see fpdt_internal.h); Q is loaded once and stays in registers.
//
// Workgroup = 4 waves; each wave owns NQ blocks of 32 query rows of one head; all waves
// share the K/V tiles staged (double-buffered) in LDS.
#include "fpdt_internal.h"
#include "mfma_tiles.h"

namespace fpdt {

namespace {

constexpr int BK = 64;          // keys per LDS tile
constexpr int KB = BK / 32;     // 32-key blocks per tile
constexpr int NWAVE = 4;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

struct FwdKernelArgs {
    const uint16_t* Q;
    const u32x4* Knat;
    const u32x4* Vtr;
    int64_t kv_head_stride_blocks;
    uint16_t* O;
    float* LSE;
    int64_t lse_stride;
    float* st_acc;
    float* st_ml;
    int64_t q_pos0, k_pos0;
    int n_q, n_keys;
    int Hq, g, flags;
    float c;  // scale * log2(e)
};

template <int D, int NQ>
__global__ __launch_bounds__(256) void fwd_sweep_kernel(FwdKernelArgs p)
{
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int BQ = NWAVE * 32 * NQ;
    constexpr int K_U4 = KB * DT * 64;      // u32x4 per K tile
    constexpr int V_U4 = KB * 2 * DB * 64;  // u32x4 per V tile
    constexpr int T_U4 = K_U4 + V_U4;
    constexpr int NLD = (T_U4 + 255) / 256;
    __shared__ u32x4 smem[2][T_U4];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int head = blockIdx.x % p.Hq;
    const int n_qt = p.n_q / BQ;
    const int qt = n_qt - 1 - (int)(blockIdx.x / p.Hq);  // heaviest (latest) tiles first
    const int kvh = head / p.g;
    const int q0 = qt * BQ;          // first row of the workgroup within the launch
    const int qw0 = q0 + w * 32 * NQ;  // first row of this wave

    // keys this workgroup needs: positions <= last query position
    const int64_t last_q_pos = p.q_pos0 + q0 + BQ - 1;
    int64_t need = last_q_pos - p.k_pos0 + 1;
    if (need > p.n_keys) need = p.n_keys;
    const int n_tiles = (int)((need + BK - 1) / BK);
    const bool may_mask = (p.k_pos0 + (int64_t)n_tiles * BK - 1) > (p.q_pos0 + q0);

    const u32x4* kbase = p.Knat + (size_t)kvh * p.kv_head_stride_blocks * (DT * 64);
    const u32x4* vbase = p.Vtr + (size_t)kvh * p.kv_head_stride_blocks * (2 * DB * 64);

    // Q fragments (B operand of S^T = K Q^T): lane (col, half) holds Q[row][16t + 8 half + e]
    bf16x8 qf[NQ][DT];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const uint16_t* qrow = p.Q + ((size_t)(qw0 + 32 * nq + col) * p.Hq + head) * D + 8 * half;
#pragma unroll
        for (int t = 0; t < DT; ++t) qf[nq][t] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * t));
    }

    floatx16 acc[NQ][DB];
    float m_run[NQ], l_run[NQ];  // l_run is this lane's partial sum (its 16 keys per block)
    const size_t wg = blockIdx.x;
    if (p.flags & SWEEP_INIT) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            m_run[nq] = -INFINITY;
            l_run[nq] = 0.f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[nq][db][r] = 0.f;
        }
    } else {
        const float* sa = p.st_acc + ((wg * NWAVE + w) * NQ) * (size_t)(DB * 16 * 64);
        const float* sm = p.st_ml + ((wg * NWAVE + w) * NQ) * (size_t)(2 * 64);
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            m_run[nq] = sm[(nq * 2 + 0) * 64 + lane];
            l_run[nq] = sm[(nq * 2 + 1) * 64 + lane];
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[nq][db][r] = sa[((nq * DB + db) * 16 + r) * 64 + lane];
        }
    }

    // ---- tile pipeline: global -> registers -> LDS, one barrier per tile ----
    u32x4 pre[NLD];
#define FPDT_GLOAD(it_)                                                            \
    {                                                                              \
        const u32x4* ksrc = kbase + (size_t)(it_) * K_U4;                          \
        const u32x4* vsrc = vbase + (size_t)(it_) * V_U4;                          \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i)                            \
        {                                                                          \
            const int idx = tid + 256 * i;                                         \
            if (256 * i + 255 < K_U4) pre[i] = ksrc[idx];                          \
            else if (256 * i >= K_U4 && 256 * i + 255 < T_U4) pre[i] = vsrc[idx - K_U4]; \
            else if (idx < T_U4) pre[i] = (idx < K_U4) ? ksrc[idx] : vsrc[idx - K_U4];   \
        }                                                                          \
    }
#define FPDT_SSTORE(buf_)                                                          \
    {                                                                              \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i)                            \
        {                                                                          \
            const int idx = tid + 256 * i;                                         \
            if (256 * i + 255 < T_U4 || idx < T_U4) smem[buf_][idx] = pre[i];      \
        }                                                                          \
    }

    if (n_tiles > 0) {
        FPDT_GLOAD(0);
        FPDT_SSTORE(0);
    }
    __syncthreads();

    const int64_t qpos_w_last = p.q_pos0 + qw0 + 32 * NQ - 1;  // last query position of this wave

    for (int it = 0; it < n_tiles; ++it) {
        const bool more = (it + 1 < n_tiles);
        if (more) FPDT_GLOAD(it + 1);
        const u32x4* ks = smem[it & 1];
        const u32x4* vs = ks + K_U4;
        const int64_t key0 = p.k_pos0 + (int64_t)it * BK;  // position of the tile's first key

        if (key0 <= qpos_w_last) {  // wave-uniform: tile not entirely above this wave's diagonal
            // ---- S^T = K Q^T for the whole tile ----
            floatx16 s[KB][NQ];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kb][nq][r] = 0.f;
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    const bf16x8 a = as_bf16x8(ks[(kb * DT + t) * 64 + lane]);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) s[kb][nq] = mfma32(a, qf[nq][t], s[kb][nq]);
                }
            }
            // ---- online softmax, one query per lane ----
            bf16x8 pf[KB][2][NQ];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                const int64_t qpos = p.q_pos0 + qw0 + 32 * nq + col;
                if (may_mask && key0 + BK - 1 > p.q_pos0 + qw0 + 32 * nq) {  // wave-uniform
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int64_t kpos = key0 + 32 * kb + 8 * (r >> 2) + 4 * half + (r & 3);
                            if (kpos > qpos) s[kb][nq][r] = -INFINITY;
                        }
                }
                float mx = s[0][nq][0];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][nq][r]);
                mx = fmaxf(mx, xor32(mx));
                const float m_new = fmaxf(m_run[nq], mx * p.c);
                // Rescale only when some query of the wave raised its maximum.
                if (__any(m_new != m_run[nq])) {
                    const float alpha = __builtin_amdgcn_exp2f(m_run[nq] - m_new);
                    l_run[nq] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[nq][db][r] *= alpha;
                    m_run[nq] = m_new;
                }
                float lsum = 0.f;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(s[kb][nq][r], p.c, -m_new));
                        s[kb][nq][r] = e;
                        lsum += e;
                    }
                    pf[kb][0][nq] = pack_half<0>(s[kb][nq]);
                    pf[kb][1][nq] = pack_half<1>(s[kb][nq]);
                }
                l_run[nq] += lsum;
            }
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const bf16x8 a = as_bf16x8(vs[((kb * 2 + s2) * DB + db) * 64 + lane]);
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq)
                            acc[nq][db] = mfma32(a, pf[kb][s2][nq], acc[nq][db]);
                    }
        }
        if (more) FPDT_SSTORE((it + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue ----
    if (p.flags & SWEEP_FINAL) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            const float l_tot = l_run[nq] + xor32(l_run[nq]);
            const float inv = 1.f / l_tot;
            const int row = qw0 + 32 * nq + col;
            uint16_t* orow = p.O + ((size_t)row * p.Hq + head) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const int d = 32 * db + 8 * a4 + 4 * half;
                    if (d < D) {
                        floatx4 v;
#pragma unroll
                        for (int b = 0; b < 4; ++b) v[b] = acc[nq][db][4 * a4 + b] * inv;
                        const bf16x4 o4 = __builtin_convertvector(v, bf16x4);
                        *reinterpret_cast<bf16x4*>(orow + d) = o4;
                    }
                }
            if (half == 0)
                p.LSE[(size_t)head * p.lse_stride + row] = (m_run[nq] + __builtin_log2f(l_tot)) * LN2;
        }
    } else {
        float* sa = p.st_acc + ((wg * NWAVE + w) * NQ) * (size_t)(DB * 16 * 64);
        float* sm = p.st_ml + ((wg * NWAVE + w) * NQ) * (size_t)(2 * 64);
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            sm[(nq * 2 + 0) * 64 + lane] = m_run[nq];
            sm[(nq * 2 + 1) * 64 + lane] = l_run[nq];
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    sa[((nq * DB + db) * 16 + r) * 64 + lane] = acc[nq][db][r];
        }
    }
}

template <int D>
constexpr int nq_for() { return 2; }

}  // namespace

int fwd_q_tile(int D) { (void)D; return NWAVE * 32 * 2; }

size_t fwd_state_acc_bytes(int64_t n_q, int Hq, int D)
{
    return (size_t)n_q * Hq * dpad(D) * sizeof(float);
}
size_t fwd_state_ml_bytes(int64_t n_q, int Hq, int D)
{
    (void)D;
    return (size_t)n_q * Hq * 2 * 2 * sizeof(float);  // (m, l) for both half-lanes of a row
}

void launch_fwd_sweep(const FwdArgs& a, hipStream_t st)
{
    FwdKernelArgs k;
    k.Q = static_cast<const uint16_t*>(a.Q);
    k.Knat = static_cast<const u32x4*>(a.Knat);
    k.Vtr = static_cast<const u32x4*>(a.Vtr);
    k.kv_head_stride_blocks = a.kv_head_stride_blocks;
    k.O = static_cast<uint16_t*>(a.O);
    k.LSE = a.LSE;
    k.lse_stride = a.lse_stride;
    k.st_acc = a.st_acc;
    k.st_ml = a.st_ml;
    k.q_pos0 = a.q_pos0;
    k.k_pos0 = a.k_pos0;
    k.n_q = (int)a.n_q;
    k.n_keys = (int)a.n_keys;
    k.Hq = a.Hq;
    k.g = a.Hq / a.Hkv;
    k.flags = a.flags;
    k.c = a.scale * LOG2E;
    const int BQ = fwd_q_tile(a.D);
    dim3 grid((unsigned)((a.n_q / BQ) * a.Hq));
    if (a.D == 128) fwd_sweep_kernel<128, 2><<<grid, 256, 0, st>>>(k);
    else if (a.D == 80) fwd_sweep_kernel<80, 2><<<grid, 256, 0, st>>>(k);
    else fwd_sweep_kernel<64, 2><<<grid, 256, 0, st>>>(k);
}

}  // namespace fpdt
