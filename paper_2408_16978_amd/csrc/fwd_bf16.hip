// Forward chunk sweep on bf16 MFMA (Sec. 4.1: query chunk against key/value chunks with
// online-softmax accumulation; causal mask only where the key range reaches the queries).
//
// Formulation: the score tile is computed transposed, S^T = K Q^T (keys are MFMA rows,
// queries are MFMA columns).  In the 32x32 accumulator layout a lane then owns ONE query
// (column lane%32) and 16 keys per 32-key block, so the running max of a query needs a single
// exchange between lanes l and l+32, the running sum none until the epilogue, and the
// exponentiated tile -- still in registers -- is directly the B operand of O^T += V^T P^T.
// K arrives as NAT fragments, V as TR fragments (fpdt_internal.h); Q is loaded once and
// stays in registers.
//
// Workgroup = 8 waves (two per SIMD, so one wave's softmax arithmetic runs under the other's
// MFMAs), each wave owns 32 query rows of one head and at most 256 registers; all waves
// share the 64-key K/V tiles, which travel global -> LDS directly (no register staging)
// through a 3-slot ring filled two tiles ahead.
#include "fpdt_internal.h"
#include "mfma_tiles.h"

namespace fpdt {

namespace {

constexpr int BK = 64;       // keys per LDS tile
constexpr int KB = BK / 32;  // 32-key blocks per tile
constexpr int NWAVE = 8;
constexpr int NTHREAD = NWAVE * 64;
constexpr int BQ = NWAVE * 32;  // query rows per workgroup
constexpr int RING = 3;
constexpr int PF = RING - 1;  // tiles in flight ahead of the one being computed
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

template <int D>
__global__ __launch_bounds__(NTHREAD) void fwd_sweep_kernel(FwdKernelArgs p)
{
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int K_U4 = KB * DT * 64;      // u32x4 per K tile
    constexpr int V_U4 = KB * 2 * DB * 64;  // u32x4 per V tile
    constexpr int T_U4 = K_U4 + V_U4;
    constexpr int KFRAG = KB * DT, NFRAG = KFRAG + KB * 2 * DB;  // 1 KiB fragments per tile
    // one LDS array per ring slot
    static_assert(RING == 3, "the tile loop below is unrolled over three slots");
    __shared__ u32x4 ring0[T_U4], ring1[T_U4], ring2[T_U4];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int half = lane >> 5, col = lane & 31;
    const int head = blockIdx.x % p.Hq;
    const int n_qt = p.n_q / BQ;
    const int qt = n_qt - 1 - (int)(blockIdx.x / p.Hq);  // heaviest (latest) tiles first
    const int kvh = head / p.g;
    const int q0 = qt * BQ;       // first row of the workgroup within the launch
    const int qw0 = q0 + w * 32;  // first row of this wave

    // keys this workgroup needs: positions <= last query position
    const int64_t last_q_pos = p.q_pos0 + q0 + BQ - 1;
    int64_t need = last_q_pos - p.k_pos0 + 1;
    if (need > p.n_keys) need = p.n_keys;
    const int n_tiles = (int)((need + BK - 1) / BK);

    const u32x4* kbase = p.Knat + (size_t)kvh * p.kv_head_stride_blocks * (DT * 64);
    const u32x4* vbase = p.Vtr + (size_t)kvh * p.kv_head_stride_blocks * (2 * DB * 64);

    // Copy tile `it` into ring slot `slot`: wave w moves fragments w, w+8, ...
    auto issue = [&](int it, u32x4* slot) {
        const u32x4* ksrc = kbase + (size_t)it * K_U4;
        const u32x4* vsrc = vbase + (size_t)it * V_U4;
#pragma unroll
        for (int f0 = 0; f0 < NFRAG; f0 += NWAVE) {
            const int f = f0 + wu;
            if (f0 + NWAVE <= NFRAG || f < NFRAG) {
                const u32x4* src = f < KFRAG ? ksrc + f * 64 : vsrc + (f - KFRAG) * 64;
                frag_to_lds(src, slot + f * 64, lane);
            }
        }
    };

    // Q fragments (B operand of S^T = K Q^T): lane (col, half) holds Q[row][16t + 8 half + e]
    bf16x8 qf[DT];
    {
        const uint16_t* qrow = p.Q + ((size_t)(qw0 + col) * p.Hq + head) * D + 8 * half;
#pragma unroll
        for (int t = 0; t < DT; ++t) qf[t] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * t));
    }

    floatx16 acc[DB];
    float m_run, l_run;  // l_run is this lane's partial sum (its 16 keys per block)
    const size_t wg = blockIdx.x;
    float* sa = p.st_acc + (wg * NWAVE + w) * (size_t)(DB * 16 * 64);
    float* sm = p.st_ml + (wg * NWAVE + w) * (size_t)(2 * 64);
    if (p.flags & SWEEP_INIT) {
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    } else {
        m_run = sm[lane];
        l_run = sm[64 + lane];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = sa[(db * 16 + r) * 64 + lane];
    }

    if (n_tiles > 0) issue(0, ring0);
    if (n_tiles > 1) issue(1, ring1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    const int64_t qpos_first = p.q_pos0 + qw0;  // first / last query position of this wave
    const int64_t qpos_last = qpos_first + 31;
    const int64_t qpos = qpos_first + col;
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One tile: compute on slot `ks`, prefetch tile it+PF into slot `pf_slot`.
    auto tile = [&](int it, const u32x4* ks, u32x4* pf_slot) {
        if (it + PF < n_tiles) issue(it + PF, pf_slot);
        const u32x4* vs = ks + K_U4;
        const int64_t key0 = p.k_pos0 + (int64_t)it * BK;  // position of the tile's first key

        if (key0 <= qpos_last) {  // wave-uniform: tile not entirely above this wave's diagonal
            // ---- S^T = K Q^T for the whole tile: all K fragments are requested up front so
            // that the MFMA chain never waits on LDS latency ----
            bf16x8 kfr[KB][DT];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int t = 0; t < DT; ++t) kfr[kb][t] = as_bf16x8(ks[(kb * DT + t) * 64 + lane]);
            floatx16 s[KB];
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) s[kb] = mfma32(kfr[kb][t], qf[t], t == 0 ? zero : s[kb]);
            __builtin_amdgcn_sched_group_barrier(0x100, KB * DT, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, KB * DT, 0);
            // V fragments are requested now and arrive under the softmax arithmetic
            bf16x8 vfr[KB][2][DB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db) vfr[kb][s2][db] = as_bf16x8(vs[((kb * 2 + s2) * DB + db) * 64 + lane]);
            __builtin_amdgcn_sched_group_barrier(0x100, KB * 2 * DB, 0);
            // ---- online softmax, one query per lane ----
            if (key0 + BK - 1 > qpos_first) {  // wave-uniform: the tile straddles the diagonal
                // key index within the tile vs this lane's query, in 32 bits: a key is masked
                // when 32 kb + 8 (r / 4) + r % 4 + 4 half > qpos - key0
                int64_t d = qpos - key0;
                d = d < -1 ? -1 : d > BK ? BK : d;
                const int rel = (int)d - 4 * half;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * kb + 8 * (r >> 2) + (r & 3) > rel) s[kb][r] = -INFINITY;
            }
            // The running maximum is only a reference point: any value gives the same O and LSE as
            // long as nothing overflows.  So the tile is exponentiated against the reference it
            // found, optimistically, and no maximum is taken at all; the row sums that are needed
            // anyway tell when that was wrong: every probability is at most the partial sum it
            // went into, so a sum within REF_LIMIT (far inside the range of bf16 and of the fp32
            // sums) proves that no probability exceeded it.  A sum beyond it -- or infinite, or not
            // a number, as on a row's first tile, where the reference is still -inf -- sends the
            // whole wave through the exact path below (true maximum, rescale, exponentiate again):
            // a row's first tile, and later only when its maximum rises by more than 14 in log2.
            constexpr float REF_LIMIT = 16384.f;
            bf16x8 pf[KB][2];
            float lsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                floatx16 e;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    e[r] = __builtin_amdgcn_exp2f(fmaf(s[kb][r], p.c, -m_run));
                    lsum += e[r];
                }
                pf[kb][0] = pack_half<0>(e);
                pf[kb][1] = pack_half<1>(e);
            }
            if (__any(!(lsum <= REF_LIMIT))) {
                float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int r = (kb == 0 ? 2 : 0); r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[kb][r]), s[kb][r + 1]);
                mx = fmaxf(mx, xor32(mx));
                const float mc = mx * p.c;
                const float m_new = mc > m_run ? mc : m_run;  // (a lane whose keys are all masked keeps its reference)
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on a row's first tile, 1 where nothing moved
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
                m_run = m_new;
                lsum = 0.f;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    floatx16 e;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        e[r] = __builtin_amdgcn_exp2f(fmaf(s[kb][r], p.c, -m_new));
                        lsum += e[r];
                    }
                    pf[kb][0] = pack_half<0>(e);
                    pf[kb][1] = pack_half<1>(e);
                }
            }
            l_run += lsum;
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        acc[db] = mfma32(vfr[kb][s2][db], pf[kb][s2], acc[db]);
        }
        // tile it+1 must have landed; the loads of tile it+PF issued above may stay in flight
        if (it + PF < n_tiles) wait_vmem_at_most<NFRAG / NWAVE>();
        else wait_vmem_at_most<0>();
        barrier_no_fence();
    };
    for (int it = 0; it < n_tiles; it += 3) {
        tile(it, ring0, ring2);
        if (it + 1 < n_tiles) tile(it + 1, ring1, ring0);
        if (it + 2 < n_tiles) tile(it + 2, ring2, ring1);
    }

    // ---- epilogue ----
    if (p.flags & SWEEP_FINAL) {
        const float l_tot = l_run + xor32(l_run);
        const float inv = 1.f / l_tot;
        const int row = qw0 + col;
        uint16_t* orow = p.O + ((size_t)row * p.Hq + head) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const int d = 32 * db + 8 * a4 + 4 * half;
                if (d < D) {
                    floatx4 v;
#pragma unroll
                    for (int b = 0; b < 4; ++b) v[b] = acc[db][4 * a4 + b] * inv;
                    *reinterpret_cast<bf16x4*>(orow + d) = __builtin_convertvector(v, bf16x4);
                }
            }
        if (half == 0) p.LSE[(size_t)head * p.lse_stride + row] = (m_run + __builtin_log2f(l_tot)) * LN2;
    } else {
        sm[lane] = m_run;
        sm[64 + lane] = l_run;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) sa[(db * 16 + r) * 64 + lane] = acc[db][r];
    }
}

}  // namespace

int fwd_q_tile(int D) { (void)D; return BQ; }

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
    dim3 grid((unsigned)((a.n_q / BQ) * a.Hq));
    if (a.D == 128) fwd_sweep_kernel<128><<<grid, NTHREAD, 0, st>>>(k);
    else if (a.D == 80) fwd_sweep_kernel<80><<<grid, NTHREAD, 0, st>>>(k);
    else fwd_sweep_kernel<64><<<grid, NTHREAD, 0, st>>>(k);
}

}  // namespace fpdt
