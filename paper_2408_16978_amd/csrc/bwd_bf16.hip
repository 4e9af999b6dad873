// Backward of the chunked attention on bf16 MFMA (Sec. 4.2; operand set of Sec. 3.1).
//
//   Delta = rowsum(dO * O)                                   (delta_kernel, HBM-bound)
//   p  = exp(scale q k^T - LSE), masked above the diagonal
//   dV += p^T dO,  dP = dO v^T,  dS = p (dP - Delta)
//   dK += scale dS^T q,  dQ += scale dS k
//
// Two MFMA kernels, each keeping its accumulators in registers and recomputing p:
//   bwd_dkdv_kernel_w4 : a workgroup (4 waves, one per SIMD) owns 256 keys of one KV head and
//       walks the query rows (all query heads of the group).  Scores are computed as S = Q K^T
//       (queries are MFMA rows, keys are columns): a lane owns one key, and the
//       register-resident p and dS tiles are the B operands of dV^T += dO^T p and
//       dK^T += Q^T dS.
//   bwd_dq_kernel      : a workgroup (8 waves, two per SIMD, at most 256 registers each, so one
//       wave's exp / dS arithmetic runs under the other's MFMAs) owns 256 query rows of one head
//       and walks the keys with S^T = K Q^T (as in the forward): a lane owns one query, LSE and
//       Delta are per-lane scalars, and dS^T is the B operand of dQ^T += K^T dS^T.
// Both stream their operands global -> LDS directly through a small ring, as NAT fragments
// (fpdt_internal.h) only: an operand whose contraction runs over rows (Q^T, dO^T, K^T) is read
// out of the same LDS block with transposing loads.
#include <type_traits>

#include "fpdt_internal.h"
#include "mfma_tiles.h"

namespace fpdt {

namespace {

constexpr int NWAVE = 8;
constexpr int NTHREAD = NWAVE * 64;
constexpr float LOG2E = 1.4426950408889634f;

struct BwdKernelArgs {
    const uint16_t* Q; const uint16_t* dO; const uint16_t* K; const uint16_t* V;
    const u32x4* Qnat; const u32x4* dOnat;
    int64_t q_head_stride_blocks;
    const u32x4* Knat; const u32x4* Vnat;
    int64_t kv_head_stride_blocks;
    const float* LSE; const float* Delta; int64_t row_stat_stride;
    const float* stat2;  // dK/dV kernel: per (head, 32-row block) 32 x LSE * log2(e), then 32 x -Delta
    int64_t q_pos0, k_pos0;
    int n_q, n_k;
    int Hq, Hkv, g, flags;
    float scale, c;
    float* acc_dq; float* acc_dk; float* acc_dv;
    uint16_t* dQ; uint16_t* dK; uint16_t* dV;
    u32x4* dS;  // dS fragments of the launch (stored-dS backward), or null
};

// Store a transposed accumulator tile set (lane = one row, registers = channels) as bf16
// into a [rows, H, D] tensor.
template <int D, int DB>
__device__ __forceinline__ void store_rows_bf16(const floatx16 (&acc)[DB], float mul, uint16_t* rowp, int half)
{
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            const int d = 32 * db + 8 * a4 + 4 * half;
            if (d < D) {
                floatx4 v;
#pragma unroll
                for (int b = 0; b < 4; ++b) v[b] = acc[db][4 * a4 + b] * mul;
                *reinterpret_cast<bf16x4*>(rowp + d) = __builtin_convertvector(v, bf16x4);
            }
        }
}

// ---------------------------------------------------------------------------------------
// dK, dV.  Wave w owns keys [k0 + 64 w, +64) (one wave per SIMD, 4 waves, 256 keys per
// workgroup): its K fragments are stationary in registers, its V fragments are parked in LDS.
// Every step stages one 32-row query block (Q, dO, LSE * log2e, -Delta) in a 2-slot LDS ring,
// loaded one step ahead.
//
// A 32-key tile per wave needs one 1 KiB LDS fragment per MFMA, which LDS cannot deliver at
// the MFMA rate; 64 keys per wave use every Q / dO fragment twice.  The dK/dV accumulator
// registers (256 at D = 128) then have to live in AGPRs while the short-lived S / dP tiles must stay in
// architectural VGPRs (VALU cannot read AGPRs): the compiler picks one form for all MFMAs of
// a function, so the MFMAs are issued through inline assembly with explicit register classes,
// and the wait states between an MFMA result and its first VALU reader, which the compiler
// inserts for the builtin, are inserted by hand (s_nop).  The step is written in the order
// it should issue: S chains | dP chains with the exp arithmetic in their shadow | dV MFMAs
// with the dS arithmetic in their shadow | dK MFMAs.
#define FPDT_MFMA_V0(d, a, b) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b))
#define FPDT_MFMA_VC(d, a, b, c) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(c))
#define FPDT_MFMA_V(d, a, b) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b))
#define FPDT_MFMA_A(d, a, b) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b))
// >= 11 wait states between an 8-pass MFMA writing a VGPR and a VALU instruction reading it
#define FPDT_MFMA_TO_VALU_NOPS() asm volatile("s_nop 7\n\ts_nop 4" ::: "memory")
#define FPDT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// STORE_DS: the rounded dS tiles, which are this kernel's own MFMA operands, are also written to
// p.dS as 1 KiB fragments [head][32-query block][32-key block][s2][lane][8]: lane (key c, h') of
// fragment s2 holds dS[q = 16 s2 + 8 (e / 4) + 4 h' + e % 4][key c], e = 0..7 -- exactly the register
// contents.  bwd_dq_ds_kernel reads them back instead of recomputing S and dP.
template <int D, bool STORE_DS>
__global__ __launch_bounds__(256) void bwd_dkdv_kernel_w4(BwdKernelArgs p)
{
    constexpr int NW = 4, NK = 2;
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int NAT_U4 = DT * 64;
    constexpr int SLOT_U4 = 2 * NAT_U4;  // Q block | dO block, each once (see "Operand layout" below)
    constexpr int NFRAG = 2 * DT;
    constexpr int RING = 2;
    constexpr int BKT = NW * 32 * NK;  // keys per workgroup
    static_assert(RING == 2, "the step loops below alternate between two slots");
    // (DP > D: the transposing loads of the padded channels reach one fragment past a block;
    // the values land in accumulator columns that are never stored, the pad keeps them in LDS)
    constexpr int SLOT_PAD = DP > D ? 64 : 0;
    constexpr int UFRAG = 2 * DT + 4 * DB;  // A-operand fragments a step consumes
    constexpr int NCOPY = (NFRAG + NW - 1) / NW;
    __shared__ u32x4 slot0[SLOT_U4 + SLOT_PAD], slot1[SLOT_U4 + SLOT_PAD];
    __shared__ u32x4 vst[NW * NK * DT * 64];  // V NAT fragments of the workgroup's keys
    __shared__ __attribute__((aligned(16))) float stat0[64], stat1[64];  // LSE*log2e | -Delta

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int half = lane >> 5, col = lane & 31;
    const int kvh = blockIdx.x % p.Hkv;
    const int kt = blockIdx.x / p.Hkv;
    const int k0 = kt * BKT, kw0 = k0 + 32 * NK * wu;
    const int64_t kpos_w0 = p.k_pos0 + kw0;

    floatx16 dk[NK][DB], dv[NK][DB];
    const size_t wg = blockIdx.x;
    float* adk = p.acc_dk + ((wg * NW + w) * NK) * (size_t)(DB * 16 * 64);
    float* adv = p.acc_dv + ((wg * NW + w) * NK) * (size_t)(DB * 16 * 64);
    if (p.flags & ACC_LOAD) {
#pragma unroll
        for (int kb = 0; kb < NK; ++kb)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    dk[kb][db][r] = adk[((kb * DB + db) * 16 + r) * 64 + lane];
                    dv[kb][db][r] = adv[((kb * DB + db) * 16 + r) * 64 + lane];
                }
                // into accumulation registers right away, one tile pair at a time: left to the
                // first MFMA that uses them, all 256 values would sit in architectural registers
                asm volatile("" : "+a"(dk[kb][db]), "+a"(dv[kb][db]));
            }
    } else {
#pragma unroll
        for (int kb = 0; kb < NK; ++kb)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int r = 0; r < 16; ++r) dk[kb][db][r] = dv[kb][db][r] = 0.f;
                asm volatile("" : "+a"(dk[kb][db]), "+a"(dv[kb][db]));
            }
    }

    // loaded after the accumulators so that nothing has to be parked in scratch across their
    // initialisation (a reload in front of the loop would put a full vector-memory wait, which
    // also covers the operand copies in flight, at its first use inside the loop)
    bf16x8 kf[NK][DT];
    u32x4* vmine = vst + wu * (NK * DT * 64);
#pragma unroll
    for (int kb = 0; kb < NK; ++kb) {
        const size_t off = ((size_t)(kw0 + 32 * kb + col) * p.Hkv + kvh) * D + 8 * half;
        const u32x4* vsrc = p.Vnat + ((size_t)kvh * p.kv_head_stride_blocks + (kw0 / 32 + kb)) * NAT_U4;
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            kf[kb][t] = as_bf16x8(*reinterpret_cast<const u32x4*>(p.K + off + 16 * t));
            frag_to_lds(vsrc + t * 64, vmine + (kb * DT + t) * 64, lane);
        }
    }

    const int64_t qmin = p.k_pos0 + k0 - p.q_pos0;
    const int qb_start = qmin > 0 ? (int)(qmin / 32) : 0;
    const int n_qb_all = p.n_q / 32;
    const int n_qb = n_qb_all > qb_start ? n_qb_all - qb_start : 0;
    const int n_iter = n_qb * p.g;
    // blocks whose first query precedes the workgroup's last key need the mask (for some wave)
    const int64_t kpos_last = p.k_pos0 + k0 + BKT - 1;
    int64_t dend = (kpos_last - p.q_pos0 + 31) / 32;
    if (dend < qb_start) dend = qb_start;
    if (dend > n_qb_all) dend = n_qb_all;
    const int n_hot_iter = (n_qb_all - (int)dend) * p.g;  // walked first (descending order)

    // Operand layout.  A step needs the 32 x D Q and dO blocks twice: as A operands contracted
    // over d (S = Q K^T, dP = dO V^T; lane = query row, 8 consecutive d) and contracted over the
    // query (dV^T += dO^T P, dK^T += Q^T dS; lane = d, 8 queries).  LDS holds each block ONCE, in
    // the first form's fragment order; the second form is read with the transposing LDS load
    // (ds_read_b64_tr_b16: each 16-lane group reads a 4-row x 16-column block of 16-bit values,
    // lane i of the group supplying the address of row i / 4, columns 4 (i % 4) .. +3, and lane j
    // receiving column j of the four rows).  That halves the copies and the LDS footprint of a
    // step.  Within fragment t (16 columns of d) the 16-byte piece (h', q) = row q, columns
    // 16 t + 8 h' .. +7 sits at position 32 h' + (q ^ 4 h' ^ 8 (t % 2)) instead of 32 h' + q: with
    // that swizzle the 32 lanes a transposing load serves per cycle hit 32 different 8-byte bank
    // pairs, and a plain fragment read is still a permutation of one contiguous KiB.
    //
    // Wave w copies fragments w, w+4, ... of the 2 D/16 that make a step (fragment f belongs to
    // operand f / (D/16); at D = 128 its parity is w's and its operand is known at compile time).
    // The copy engine writes lane l's 16 bytes at position l, so lane l fetches the piece that
    // belongs there.  The copies of a wave are NOT issued back
    // to back: the CU's address unit takes them one at a time, and a wave whose copy is not
    // accepted yet cannot issue its next MFMA either.  issue_begin() sets up the addresses (and
    // requests the row statistics), issue_one() sends one copy; a step calls it between its first
    // MFMA groups.
    uint64_t cp_src[2] = {0, 0};  // scalar registers: this wave's first fragment of each operand
    uint64_t stat_src = 0;
    uint64_t ds_next = 0;  // (STORE_DS) where the step that issue_begin() was last called for stores its dS fragments
    const unsigned stat_addr[2] = {lds_address(stat0), lds_address(stat1)};
    // (DT even: the parity of every fragment a wave copies is the wave's; DT odd: chosen per copy)
    const int cp_lane_par[2] = {16 * (32 * half + (col ^ (4 * half))), 16 * (32 * half + (col ^ (4 * half) ^ 8))};
    const int cp_lane_off = cp_lane_par[wu & 1];
    const unsigned slot_addr[2] = {lds_address(slot0), lds_address(slot1)};
    const unsigned slot_lds[2] = {slot_addr[0] + 1024u * (unsigned)wu, slot_addr[1] + 1024u * (unsigned)wu};
    // positions of this lane's piece in an even / odd fragment (plain fragment reads)
    const int natpos[2] = {32 * half + (col ^ (4 * half)), 32 * half + (col ^ (4 * half) ^ 8)};
    // byte offsets of this lane's two transposing loads within a block (first / second group of
    // four queries), to which 2048 db + 256 s2 is added for the fragment (32 db + .. d, 16 s2 + .. q)
    int trb[2];
    {
        const int grp = lane >> 4, i16 = lane & 15, e = i16 >> 2, x = i16 & 3;
        const int h = grp >> 1, dblk = grp & 1, hq = x >> 1;
#pragma unroll
        for (int I = 0; I < 2; ++I)
            trb[I] = 1024 * dblk + 512 * hq + 16 * (e + 4 * (h ^ hq) + 8 * (I ^ dblk)) + 8 * (x & 1);
    }
    // issue_begin(it) sets the scalar source addresses of step `it`: block (head, qb) with
    // hh = it % g, qb = n_qb_all - 1 - it / g, head = kvh g + hh.  It is called for it = 0, 1, 2, ..
    // in order (and once more for the last step), so the addresses are advanced by one of two
    // precomputed strides instead of being rebuilt: no division, no vector instruction, a dozen
    // scalar instructions at the head of a step, where nothing hides them.
    const int w64 = DT == 8 ? wu * 64 : 0;  // D = 128: the wave's first fragment of each operand
    const int64_t blk_next_head = p.q_head_stride_blocks;                          // hh + 1, same qb
    const int64_t blk_next_qb = -(int64_t)(p.g - 1) * p.q_head_stride_blocks - 1;  // hh wraps to 0, qb - 1
    const int64_t pair_next_head = (int64_t)n_qb_all * (p.n_k / 32);
    const int64_t pair_next_qb = -(int64_t)(p.g - 1) * pair_next_head - (p.n_k / 32);
    int st_it = 0, st_hh = 0;  // the step the addresses below belong to, and its head within the group
    {
        const int64_t blk0 = (int64_t)(kvh * p.g) * p.q_head_stride_blocks + (n_qb_all - 1);
        cp_src[0] = (uint64_t)(uintptr_t)(p.Qnat + blk0 * NAT_U4 + w64);
        cp_src[1] = (uint64_t)(uintptr_t)(p.dOnat + blk0 * NAT_U4 + w64);
        stat_src = (uint64_t)(uintptr_t)(p.stat2 + blk0 * 64);
        if constexpr (STORE_DS) {
            // fragment pairs (head, query block, key block) of a launch are fewer than 2^31 (API layer)
            const int64_t pair0 = ((int64_t)(kvh * p.g) * n_qb_all + (n_qb_all - 1)) * (p.n_k / 32) + kw0 / 32;
            ds_next = (uint64_t)(uintptr_t)p.dS + ((uint64_t)pair0 << 11);
        }
    }
    auto issue_begin = [&](int it) {
        if (it == st_it) return;  // the first step, and the last step's second request
        st_it = it;
        const bool wrap = ++st_hh == p.g;
        if (wrap) st_hh = 0;
        const int64_t db = wrap ? blk_next_qb : blk_next_head;
        cp_src[0] += (uint64_t)(db * (int64_t)(NAT_U4 * 16));
        cp_src[1] += (uint64_t)(db * (int64_t)(NAT_U4 * 16));
        // the block's row statistics (256 bytes, already in the form the step consumes) travel
        // through the copy engine like the operands: no vector register, no wait of the compiler's
        stat_src += (uint64_t)(db * 256);
        if constexpr (STORE_DS) ds_next += (uint64_t)((wrap ? pair_next_qb : pair_next_head) * 2048);
    };
    // k = 0..3 (compile-time after unrolling): fragment 4 k + w of the step, i.e. fragment
    // 4 (k % 2) + w of operand k / 2; into_slot1 is a compile-time constant at every call
    auto issue_one = [&](int k, bool into_slot1) {
        if (k == 0 && wu == 0) dwords_to_lds_at(stat_src, stat_addr[into_slot1], lane * 4);
        if constexpr (DT == 8) {
            frag_to_lds_at(cp_src[k / 2] + 1024u * (unsigned)(NW * (k % 2)), slot_lds[into_slot1] + 1024u * (unsigned)(NW * k), cp_lane_off);
        } else {
            // fragment f of the step (operand f / DT, its fragment f % DT); a wave without a
            // fragment in the last round copies its previous one again (same bytes, same place)
            int f = NW * k + wu;
            if (f >= NFRAG) f -= NW;
            const int op = f >= DT ? 1 : 0, t = f - op * DT;
            const uint64_t src = (op ? cp_src[1] : cp_src[0]) + 1024u * (unsigned)t;
            frag_to_lds_at(src, slot_addr[into_slot1] + 1024u * (unsigned)f, cp_lane_par[0] ^ (128 * (t & 1)));
        }
    };
    auto issue = [&](int it, bool into_slot1) {
        issue_begin(it);
#pragma unroll
        for (int k = 0; k < NCOPY; ++k) issue_one(k, into_slot1);
    };

    // One step.  The 32 A-operand fragments are consumed in the order Q 0..7, dO 0..7 (plain),
    // dO^T 0..7, Q^T 0..7 (transposing loads); they are read from LDS four MFMA pairs ahead into
    // a ring of six registers sets, so that a set is overwritten only two pairs after its last
    // reader was issued.
    typedef short short4v __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;
    auto step = [&](auto masked_tag, int it, const u32x4* sl, const float* st, u32x4* nslot, float* nst) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        (void)nst;  // filled by the copy that issue_one(0, ..) sends with the next step's operands
        const uint64_t ds_dst = ds_next;  // set when this step's operands were requested
        const bool more = it + 1 < n_iter;
        // the last step copies its own operands once more into the idle slot: the copies in the
        // MFMA sequence below then need no branch around them
        issue_begin(more ? it + 1 : it);
        if (MASKED) {  // diagonal steps (few): a wave may skip the arithmetic, so all copies go first
#pragma unroll
            for (int k = 0; k < NCOPY; ++k) issue_one(k, nslot == slot1);
        }
        const int qb = n_qb_all - 1 - it / p.g;
        const int64_t qpos_b0 = p.q_pos0 + (int64_t)qb * 32;

        if (!MASKED || qpos_b0 + 31 >= kpos_w0) {  // wave-uniform
            const unsigned sl_addr = slot_addr[sl == slot1];
            const unsigned tr0 = sl_addr + (unsigned)trb[0], tr1 = sl_addr + (unsigned)trb[1];
            // fragment u of the stream: 0..15 plain (Q | dO), 16..23 dO^T, 24..31 Q^T
            auto afrag = [&](int u) -> bf16x8 {
                if (u < 2 * DT) return as_bf16x8(sl[u * 64 + natpos[(u % DT) & 1]]);
                const bool of_dO = u < 2 * DT + 2 * DB;
                const int i = of_dO ? u - 2 * DT : u - 2 * DT - 2 * DB;
                const unsigned o = (of_dO ? 1024u * DT : 0u) + 2048u * (unsigned)(i % DB) + 256u * (unsigned)(i / DB);
                const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)(tr0 + o));
                const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)(tr1 + o));
                typedef short short8v __attribute__((ext_vector_type(8)));
                const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(bf16x8, both);
            };
#define FPDT_AFRAG(u_) afrag(u_)
            bf16x8 fr[6], vb0[3], vb1[3];
#pragma unroll
            for (int u = 0; u < 4; ++u) fr[u] = FPDT_AFRAG(u);
            vb0[0] = as_bf16x8(vmine[(0 * DT + 0) * 64 + lane]);
            vb1[0] = as_bf16x8(vmine[(1 * DT + 0) * 64 + lane]);
            floatx16 s0, s1, dp0, dp1;
            bf16x8 pf[NK][2], df[NK][2];
            // per-row statistics are read one chunk ahead of their use and BEFORE the fragment
            // reads of that chunk, so the wait in front of the arithmetic never includes a
            // 1 KiB fragment read (LDS returns in order)
            auto stat2 = [&](int base, int r) {  // rows r, r+1 (r even): consecutive floats
                return *reinterpret_cast<const float2*>(st + base + 8 * (r >> 2) + 4 * half + (r & 3));
            };
            // The dP chains start from the tile of -Delta instead of zero (registers 4a .. 4a+3
            // hold rows 8a + 4 half + 0..3: four 16-byte reads), so the MFMAs deliver dP - Delta
            // and the dS arithmetic loses its subtraction.
            floatx16 nd;
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const floatx4 q4 = *reinterpret_cast<const floatx4*>(st + 32 + 8 * a4 + 4 * half);
#pragma unroll
                for (int b = 0; b < 4; ++b) nd[4 * a4 + b] = q4[b];
            }
            float2 stat_nx = stat2(0, 0);
            // ---- A: S = Q K^T, two chains ----
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const int u = t;
                if (t == 0) {
                    FPDT_MFMA_V0(s0, fr[u % 6], kf[0][t]);
                    FPDT_MFMA_V0(s1, fr[u % 6], kf[1][t]);
                } else {
                    FPDT_MFMA_V(s0, fr[u % 6], kf[0][t]);
                    FPDT_MFMA_V(s1, fr[u % 6], kf[1][t]);
                }
                fr[(u + 4) % 6] = FPDT_AFRAG(u + 4);
                if (!MASKED && t % 2 == 0 && t / 2 < NCOPY) issue_one(t / 2, nslot == slot1);  // a copy for the next step every second MFMA pair
                FPDT_SCHED_FENCE();
            }
            // ---- B: dP - Delta = dO V^T - Delta, exp of S in the shadow of the MFMAs ----
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const int u = DT + t;
                float2 lse = stat_nx;
                if (DT == 8 && t + 1 < DT) stat_nx = stat2(0, 2 * t + 2);
                if (t == 0) {
                    FPDT_MFMA_VC(dp0, fr[u % 6], vb0[t % 3], nd);
                    FPDT_MFMA_VC(dp1, fr[u % 6], vb1[t % 3], nd);
                    FPDT_MFMA_TO_VALU_NOPS();  // s0, s1 are complete and readable from here on
                } else {
                    FPDT_MFMA_V(dp0, fr[u % 6], vb0[t % 3]);
                    FPDT_MFMA_V(dp1, fr[u % 6], vb1[t % 3]);
                }
                fr[(u + 4) % 6] = FPDT_AFRAG(u + 4);
                if (t + 1 < DT) {
                    vb0[(t + 1) % 3] = as_bf16x8(vmine[(0 * DT + t + 1) * 64 + lane]);
                    vb1[(t + 1) % 3] = as_bf16x8(vmine[(1 * DT + t + 1) * 64 + lane]);
                }
                FPDT_SCHED_FENCE();
#pragma unroll
                for (int r = 16 * t / DT; r < 16 * (t + 1) / DT; ++r) {
                    if (DT != 8 && (r % 2 == 0 || r == 16 * t / DT)) lse = stat2(0, r & ~1);  // read at use
                    const float lse2 = (r & 1) ? lse.y : lse.x;
                    float e0 = __builtin_amdgcn_exp2f(fmaf(s0[r], p.c, -lse2));
                    float e1 = __builtin_amdgcn_exp2f(fmaf(s1[r], p.c, -lse2));
                    if (MASKED) {
                        const int64_t qp = qpos_b0 + 8 * (r >> 2) + 4 * half + (r & 3);
                        if (kpos_w0 + col > qp) e0 = 0.f;
                        if (kpos_w0 + 32 + col > qp) e1 = 0.f;
                    }
                    s0[r] = e0;
                    s1[r] = e1;
                }
                if (16 * (t + 1) / DT >= 8 && 16 * t / DT < 8) {  // rows 0..7 are final
                    pf[0][0] = pack_half<0>(s0);
                    pf[1][0] = pack_half<0>(s1);
                }
                FPDT_SCHED_FENCE();
            }
            pf[0][1] = pack_half<1>(s0);
            pf[1][1] = pack_half<1>(s1);
            FPDT_SCHED_FENCE();
            // ---- C: dV^T += dO^T p, dS = p (dP - Delta) in the shadow (dp holds dP - Delta) ----
#pragma unroll
            for (int i = 0; i < 2 * DB; ++i) {
                const int u = 2 * DT + i;
                const int s2 = i / DB, db = i % DB;
                FPDT_MFMA_A(dv[0][db], fr[u % 6], pf[0][s2]);
                FPDT_MFMA_A(dv[1][db], fr[u % 6], pf[1][s2]);
                if (i == 0) FPDT_MFMA_TO_VALU_NOPS();  // dp0, dp1 readable
                fr[(u + 4) % 6] = FPDT_AFRAG(u + 4);
                FPDT_SCHED_FENCE();
#pragma unroll
                for (int r = 16 * i / (2 * DB); r < 16 * (i + 1) / (2 * DB); ++r) {
                    dp0[r] = s0[r] * dp0[r];
                    dp1[r] = s1[r] * dp1[r];
                }
                if (16 * (i + 1) / (2 * DB) >= 8 && 16 * i / (2 * DB) < 8) {  // rows 0..7 are final
                    df[0][0] = pack_half<0>(dp0);
                    df[1][0] = pack_half<0>(dp1);
                }
                FPDT_SCHED_FENCE();
            }
            df[0][1] = pack_half<1>(dp0);
            df[1][1] = pack_half<1>(dp1);
            FPDT_SCHED_FENCE();
            // ---- D: dK^T += Q^T dS ----
            if constexpr (STORE_DS && !MASKED) {
                // In the unmasked steps (all but a few per launch) the next step's operand copies are
                // waited for HERE, in front of this step's dS stores, not at the end of the step:
                // vector-memory stores and loads complete out of order with each other, so a wait that
                // has to cover the copies would cover the stores as well, and those have been in
                // flight for a quarter of a step only.  Issued now, the stores have a whole step to
                // drain.  (Compile-time choice: a run-time condition around the closing wait makes the
                // register allocator spill the accumulators.)
                wait_vmem_at_most<0>();
            }
#pragma unroll
            for (int i = 0; i < 2 * DB; ++i) {
                const int u = 2 * DT + 2 * DB + i;
                const int s2 = i / DB, db = i % DB;
                FPDT_MFMA_A(dk[0][db], fr[u % 6], df[0][s2]);
                FPDT_MFMA_A(dk[1][db], fr[u % 6], df[1][s2]);
                if (u + 4 < UFRAG) fr[(u + 4) % 6] = FPDT_AFRAG(u + 4);
                if constexpr (STORE_DS) {
                    // four 1 KiB stores spread over the MFMA pairs of this phase (issued behind the
                    // step's last MFMA instead, in the shadow of the barrier: 265 against 260 ms):
                    // fragment (kb, s2) of this step at [.. + kb][s2]; non-temporal, they are read
                    // back once by another kernel
                    constexpr int EVERY = 2 * DB >= 8 ? 2 : 1;
                    if (i % EVERY == 0 && i / EVERY < 4) {
                        const int f = i / EVERY;
                        uint64_t addr;  // address through a scalar move: copy_address_rule in mfma_tiles.h
                        asm volatile("s_mov_b64 %0, %3\n\tglobal_store_dwordx4 %1, %2, %0 nt"
                                     : "=&s"(addr)
                                     : "v"(lane * 16), "v"(__builtin_bit_cast(u32x4, df[f / 2][f % 2])),
                                       "s"(ds_dst + 1024u * (unsigned)f)
                                     : "memory");
                    }
                }
                FPDT_SCHED_FENCE();
            }
#undef FPDT_AFRAG
        }
        if constexpr (!STORE_DS || MASKED) wait_vmem_at_most<0>();  // the direct-to-LDS loads of step it+1 have landed
        barrier_no_fence();
    };

    if (n_iter > 0) issue(0, false);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // Touch the stationary K fragments in front of each loop: whatever the register allocator
    // parked in scratch is reloaded and waited for HERE; a reload whose first use is inside the
    // loop would put a full vector-memory wait (operand copies in flight included) in every step.
    auto pin_kf = [&]() {
#pragma unroll
        for (int kb = 0; kb < NK; ++kb)
#pragma unroll
            for (int t = 0; t < DT; ++t) asm volatile("" ::"v"(kf[kb][t]));
    };
    // the unmasked steps come first (descending walk); an odd count leaves the ring on slot 1
    const int n_hot_even = n_hot_iter & ~1;
    pin_kf();
    for (int it = 0; it < n_hot_even; it += 2) {
        step(std::false_type{}, it, slot0, stat0, slot1, stat1);
        step(std::false_type{}, it + 1, slot1, stat1, slot0, stat0);
    }
    pin_kf();
    for (int it = n_hot_even; it < n_iter; it += 2) {
        step(std::true_type{}, it, slot0, stat0, slot1, stat1);
        if (it + 1 < n_iter) step(std::true_type{}, it + 1, slot1, stat1, slot0, stat0);
    }

    // the accumulators are read by ordinary instructions from here on
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    if (p.flags & ACC_FINAL) {
#pragma unroll
        for (int kb = 0; kb < NK; ++kb) {
            const size_t off = ((size_t)(kw0 + 32 * kb + col) * p.Hkv + kvh) * D;
            store_rows_bf16<D, DB>(dk[kb], p.scale, p.dK + off, half);
            store_rows_bf16<D, DB>(dv[kb], 1.f, p.dV + off, half);
        }
    } else {
#pragma unroll
        for (int kb = 0; kb < NK; ++kb)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    adk[((kb * DB + db) * 16 + r) * 64 + lane] = dk[kb][db][r];
                    adv[((kb * DB + db) * 16 + r) * 64 + lane] = dv[kb][db][r];
                }
    }
}

// ---------------------------------------------------------------------------------------
// dQ.  Wave w owns query rows [q0 + 32 w, +32) of one head (Q and dO fragments, LSE and Delta
// stationary in registers).  Every step stages a 64-key tile (K-NAT, V-NAT, K-TR) in a 3-slot
// LDS ring, loaded two tiles ahead.
template <int D>
__global__ __launch_bounds__(NTHREAD) void bwd_dq_kernel(BwdKernelArgs p)
{
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int BK = 64, KB = BK / 32;
    constexpr int BQ = NWAVE * 32;
    constexpr int NAT_U4 = KB * DT * 64;  // per tile of BK keys
    // The K tile is staged once; the key-contracted operand of dQ^T += K^T dS^T is read from the
    // same block with transposing LDS loads (layout and swizzle as in the dK/dV kernel above,
    // keys in the place of queries).  With DP > D the loads of the padded channels reach into the
    // next fragments of the slot; they only feed accumulator columns that are never stored.
    constexpr int SLOT_U4 = 2 * NAT_U4;
    constexpr int NATF = KB * DT, NFRAG = 2 * NATF;
    constexpr int RING = 3;
    static_assert(RING == 3, "the tile loop below is unrolled over three slots");
    __shared__ u32x4 ring0[SLOT_U4], ring1[SLOT_U4], ring2[SLOT_U4];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int half = lane >> 5, col = lane & 31;
    const int head = blockIdx.x % p.Hq;
    const int n_qt = p.n_q / BQ;
    const int qt = n_qt - 1 - (int)(blockIdx.x / p.Hq);
    const int kvh = head / p.g;
    const int q0 = qt * BQ, qw0 = q0 + w * 32;

    const int64_t last_q_pos = p.q_pos0 + q0 + BQ - 1;
    int64_t need = last_q_pos - p.k_pos0 + 1;
    if (need > p.n_k) need = p.n_k;
    if (need < 0) need = 0;
    const int n_tiles = (int)((need + BK - 1) / BK);

    const u32x4* knb = p.Knat + (size_t)kvh * p.kv_head_stride_blocks * (DT * 64);
    const u32x4* vnb = p.Vnat + (size_t)kvh * p.kv_head_stride_blocks * (DT * 64);

    const int cp_lane0 = 32 * half + (col ^ (4 * half));  // even fragment; odd: ^ 8
    const int natpos[2] = {32 * half + (col ^ (4 * half)), 32 * half + (col ^ (4 * half) ^ 8)};
    int trb[2];  // byte offsets of this lane's two transposing loads within a 32-key block
    {
        const int grp = lane >> 4, i16 = lane & 15, e = i16 >> 2, x = i16 & 3;
        const int h = grp >> 1, dblk = grp & 1, hq = x >> 1;
#pragma unroll
        for (int I = 0; I < 2; ++I)
            trb[I] = 1024 * dblk + 512 * hq + 16 * (e + 4 * (h ^ hq) + 8 * (I ^ dblk)) + 8 * (x & 1);
    }
    typedef short short4v __attribute__((ext_vector_type(4)));
    typedef short short8v __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;
    auto issue = [&](int it, u32x4* slot) {
#pragma unroll
        for (int f0 = 0; f0 < NFRAG; f0 += NWAVE) {
            const int f = f0 + wu;
            if (f0 + NWAVE <= NFRAG || f < NFRAG) {
                const u32x4* src = f < NATF ? knb + (size_t)it * NAT_U4 + f * 64 : vnb + (size_t)it * NAT_U4 + (f - NATF) * 64;
                // a K fragment's 16-byte pieces land swizzled by the parity of its index within
                // the key block (DT even: that is the wave's parity)
                const int par = DT % 2 == 0 ? (wu & 1) : ((f % DT) & 1);
                frag_to_lds(src, slot + f * 64, f < NATF ? (cp_lane0 ^ (8 * par)) : lane);
            }
        }
    };

    bf16x8 qf[DT], of[DT];
    const int row = qw0 + col;
    {
        const size_t off = ((size_t)row * p.Hq + head) * D + 8 * half;
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            qf[t] = as_bf16x8(*reinterpret_cast<const u32x4*>(p.Q + off + 16 * t));
            of[t] = as_bf16x8(*reinterpret_cast<const u32x4*>(p.dO + off + 16 * t));
        }
    }
    const float lse2 = p.LSE[(size_t)head * p.row_stat_stride + row] * LOG2E;
    // The dP chain starts from -Delta instead of zero, so the MFMAs deliver dP - Delta directly
    // (one vector instruction per element less; plain vector instructions take issue slots from
    // the MFMAs of the SIMD's other wave).  The same trick for the scores would need Q held
    // pre-multiplied by scale * log2(e) in bf16: measured, that rounding alone pushes dQ past its
    // error budget (the cancellation in p (dP - Delta) amplifies it), so the scores keep their
    // fp32 multiply-add.
    floatx16 neg_delta;
    {
        const float dl = -p.Delta[(size_t)head * p.row_stat_stride + row];
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_delta[r] = dl;
    }

    floatx16 acc[DB];
    const size_t wg = blockIdx.x;
    float* aq = p.acc_dq + (wg * NWAVE + w) * (size_t)(DB * 16 * 64);
    if (p.flags & ACC_LOAD) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = aq[(db * 16 + r) * 64 + lane];
    } else {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    }

    if (n_tiles > 0) issue(0, ring0);
    if (n_tiles > 1) issue(1, ring1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    const int64_t qpos_first = p.q_pos0 + qw0, qpos_last = qpos_first + 31, qpos = qpos_first + col;
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // One tile: compute on slot `kn`, prefetch tile it+2 into slot `pf_slot`.
    auto tile = [&](int it, const u32x4* kn, u32x4* pf_slot) {
        if (it + 2 < n_tiles) issue(it + 2, pf_slot);
        const u32x4* vn = kn + NAT_U4;
        const unsigned kn_addr = lds_address(kn);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int64_t key0 = p.k_pos0 + (int64_t)it * BK + 32 * kb;
            if (key0 <= qpos_last) {  // wave-uniform
                // K fragments first; the V fragments are requested one per score MFMA (each has
                // the rest of the chain in front of its first use), the K-TR fragments after the
                // dP chain: they arrive under the exp2 / multiply arithmetic.  No more than two
                // fragment sets are live at a time.
                bf16x8 kfr[DT], vfr[DT], tfr[2][DB];
#pragma unroll
                for (int t = 0; t < DT; ++t) kfr[t] = as_bf16x8(kn[(kb * DT + t) * 64 + natpos[t & 1]]);
                floatx16 s, dp;
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    s = mfma32(kfr[t], qf[t], t == 0 ? zero : s);
                    vfr[t] = as_bf16x8(vn[(kb * DT + t) * 64 + lane]);
                }
#pragma unroll
                for (int t = 0; t < DT; ++t) dp = mfma32(vfr[t], of[t], t == 0 ? neg_delta : dp);
                __builtin_amdgcn_sched_group_barrier(0x100, DT, 0);
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, DT, 0);
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const unsigned o = kn_addr + 16u * 64u * (unsigned)(kb * DT) + 2048u * (unsigned)db + 256u * (unsigned)s2;
                        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)(o + (unsigned)trb[0]));
                        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)(o + (unsigned)trb[1]));
                        const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        tfr[s2][db] = __builtin_bit_cast(bf16x8, both);
                    }
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], p.c, -lse2));
                if (key0 + 31 > qpos_first) {  // wave-uniform: the block straddles the diagonal
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (key0 + 8 * (r >> 2) + 4 * half + (r & 3) > qpos) s[r] = 0.f;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) dp[r] = s[r] * dp[r];
                const bf16x8 df0 = pack_half<0>(dp), df1 = pack_half<1>(dp);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    acc[db] = mfma32(tfr[0][db], df0, acc[db]);
                    acc[db] = mfma32(tfr[1][db], df1, acc[db]);
                }
            }
        }
        // tile it+1 must have landed; the loads of tile it+2 issued above may stay in flight
        if (it + 2 < n_tiles) wait_vmem_at_most<NFRAG / NWAVE>();
        else wait_vmem_at_most<0>();
        barrier_no_fence();
    };
    for (int it = 0; it < n_tiles; it += 3) {
        tile(it, ring0, ring2);
        if (it + 1 < n_tiles) tile(it + 1, ring1, ring0);
        if (it + 2 < n_tiles) tile(it + 2, ring2, ring1);
    }

    if (p.flags & ACC_FINAL) {
        store_rows_bf16<D, DB>(acc, p.scale, p.dQ + ((size_t)row * p.Hq + head) * D, half);
    } else {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) aq[(db * 16 + r) * 64 + lane] = acc[db][r];
    }
}

// ---------------------------------------------------------------------------------------
// dQ from stored dS (the stored-dS backward).  The dK/dV kernel has written the rounded dS tiles
// of the launch; dQ^T += K^T dS^T is then ONE GEMM per chunk pair instead of three (no S, no dP,
// no exp).  Per chunk pair the tiles are n_q * n_k * Hq * 2 bytes, read once from HBM, which is
// what bounds this kernel; its MFMA work is a third of bwd_dq_kernel's.
//
// Workgroup = 8 waves x 32 query rows of one head, as in bwd_dq_kernel.  Per 64-key tile the
// K-NAT block is staged once for all waves (same layout, swizzle and transposing loads as above)
// and every wave stages the four dS fragments (2 key blocks x 2 query halves) of ITS query block.
// A stored fragment holds, per key, eight queries; the B operand of dQ^T += K^T dS^T wants, per
// query, eight keys: the same transposing LDS load delivers that (4 keys x 16 queries per 16-lane
// group and load).  The 16-byte piece of writer lane (key c, h') of fragment s2 is placed at
// position 32 h' + (c ^ 4 h' ^ 8 s2) by the copy's per-lane source address, so that the 32 lanes
// one load serves per cycle touch 32 different 8-byte bank pairs.
template <int D>
__global__ __launch_bounds__(NTHREAD) void bwd_dq_ds_kernel(BwdKernelArgs p)
{
    constexpr int DT = D / 16, DP = (D + 31) / 32 * 32, DB = DP / 32;
    constexpr int BK = 64, KB = BK / 32;
    constexpr int BQ = NWAVE * 32;
    constexpr int NATF = KB * DT;            // K fragments per tile (shared by the workgroup)
    constexpr int K_U4 = NATF * 64;
    constexpr int K_PAD = DP > D ? 64 : 0;   // transposing loads of padded channels reach past the block
    constexpr int DSF = KB * 2;              // dS fragments per tile and wave
    constexpr int DS_U4 = DSF * 64;
    constexpr int RING = 3;
    static_assert(RING == 3, "the tile loop below is unrolled over three slots");
    __shared__ u32x4 kring0[K_U4 + K_PAD], kring1[K_U4 + K_PAD], kring2[K_U4 + K_PAD];
    __shared__ u32x4 dring0[NWAVE * DS_U4], dring1[NWAVE * DS_U4], dring2[NWAVE * DS_U4];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int half = lane >> 5, col = lane & 31;
    const int head = blockIdx.x % p.Hq;
    const int n_qt = p.n_q / BQ;
    const int qt = n_qt - 1 - (int)(blockIdx.x / p.Hq);
    const int kvh = head / p.g;
    const int q0 = qt * BQ, qw0 = q0 + w * 32;

    const int64_t last_q_pos = p.q_pos0 + q0 + BQ - 1;
    int64_t need = last_q_pos - p.k_pos0 + 1;
    if (need > p.n_k) need = p.n_k;
    if (need < 0) need = 0;
    const int n_tiles = (int)((need + BK - 1) / BK);

    const u32x4* knb = p.Knat + (size_t)kvh * p.kv_head_stride_blocks * (DT * 64);
    // this wave's dS fragments: [head][query block][key block][s2][64 lanes]
    const u32x4* dsb = p.dS + (((size_t)head * (unsigned)(p.n_q / 32) + (unsigned)(q0 / 32 + wu)) * (unsigned)(p.n_k / 32)) * 128;

    const int cp_lane0 = 32 * half + (col ^ (4 * half));  // K fragments: even index within the key block; odd: ^ 8
    int trb[2];  // K^T: byte offsets of this lane's two transposing loads within a 32-key block
    int dsb_off[2];  // dS^T: the same for the wave's dS fragments of one key block
    {
        const int grp = lane >> 4, i16 = lane & 15, e = i16 >> 2, x = i16 & 3;
        const int h = grp >> 1, dblk = grp & 1, hq = x >> 1;
#pragma unroll
        for (int I = 0; I < 2; ++I)
            trb[I] = 1024 * dblk + 512 * hq + 16 * (e + 4 * (h ^ hq) + 8 * (I ^ dblk)) + 8 * (x & 1);
        // group (h, s2 = query half); lane i16 supplies row r = i16 / 4 (a key) and piece m = i16 % 4:
        // writer half h' = m % 2, upper or lower 8 bytes m / 2.  Keys of a 16-key step come in the
        // order 8 I + 4 h + r, the row order of the K^T operand above.
        const int s2 = grp & 1, r = i16 >> 2, m = i16 & 3, hw = m & 1, up = m >> 1;
#pragma unroll
        for (int I = 0; I < 2; ++I)
            dsb_off[I] = 1024 * s2 + 16 * (32 * hw + 8 * (I ^ s2) + 4 * (h ^ hw) + r) + 8 * up;
    }
    typedef short short4v __attribute__((ext_vector_type(4)));
    typedef short short8v __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;
    auto tr_frag = [&](unsigned a0, unsigned a1) -> bf16x8 {
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)a0);
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)a1);
        const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    };
    // source piece of this lane's LDS position in a dS fragment of query half s2
    const int ds_src[2] = {32 * half + (col ^ (4 * half)), 32 * half + (col ^ (4 * half) ^ 8)};
    auto issue = [&](int it, u32x4* kslot, u32x4* dslot) {
#pragma unroll
        for (int f0 = 0; f0 < NATF; f0 += NWAVE) {
            const int f = f0 + wu;
            if (f0 + NWAVE <= NATF || f < NATF) {
                const int par = DT % 2 == 0 ? (wu & 1) : ((f % DT) & 1);
                frag_to_lds(knb + (size_t)it * K_U4 + f * 64, kslot + f * 64, cp_lane0 ^ (8 * par));
            }
        }
        u32x4* mine = dslot + wu * DS_U4;
#pragma unroll
        for (int f = 0; f < DSF; ++f) frag_to_lds_nt(dsb + ((size_t)it * DSF + f) * 64, mine + f * 64, ds_src[f & 1]);
    };

    floatx16 acc[DB];
    const size_t wg = blockIdx.x;
    float* aq = p.acc_dq + (wg * NWAVE + w) * (size_t)(DB * 16 * 64);
    if (p.flags & ACC_LOAD) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = aq[(db * 16 + r) * 64 + lane];
    } else {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    }

    if (n_tiles > 0) issue(0, kring0, dring0);
    if (n_tiles > 1) issue(1, kring1, dring1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    const int64_t qpos_last = p.q_pos0 + qw0 + 31;
    constexpr int NCOPY = NATF / NWAVE + DSF;  // copies EVERY wave issues per tile (some issue one more)
    auto tile = [&](int it, const u32x4* kn, const u32x4* dsl, u32x4* pf_k, u32x4* pf_d) {
        if (it + 2 < n_tiles) issue(it + 2, pf_k, pf_d);
        const unsigned kn_addr = lds_address(kn);
        const unsigned ds_addr = lds_address(dsl + wu * DS_U4);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int64_t key0 = p.k_pos0 + (int64_t)it * BK + 32 * kb;
            if (key0 <= qpos_last) {  // wave-uniform: the dK/dV kernel wrote exactly these blocks
                bf16x8 bfr[2], tfr[2][DB];
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const unsigned o = ds_addr + 2048u * (unsigned)kb + 256u * (unsigned)s2;
                    bfr[s2] = tr_frag(o + (unsigned)dsb_off[0], o + (unsigned)dsb_off[1]);
                }
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const unsigned o = kn_addr + 16u * 64u * (unsigned)(kb * DT) + 2048u * (unsigned)db + 256u * (unsigned)s2;
                        tfr[s2][db] = tr_frag(o + (unsigned)trb[0], o + (unsigned)trb[1]);
                    }
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    acc[db] = mfma32(tfr[0][db], bfr[0], acc[db]);
                    acc[db] = mfma32(tfr[1][db], bfr[1], acc[db]);
                }
            }
        }
        if (it + 2 < n_tiles) wait_vmem_at_most<NCOPY>();
        else wait_vmem_at_most<0>();
        barrier_no_fence();
    };
    for (int it = 0; it < n_tiles; it += 3) {
        tile(it, kring0, dring0, kring2, dring2);
        if (it + 1 < n_tiles) tile(it + 1, kring1, dring1, kring0, dring0);
        if (it + 2 < n_tiles) tile(it + 2, kring2, dring2, kring1, dring1);
    }

    const int row = qw0 + col;
    if (p.flags & ACC_FINAL) {
        store_rows_bf16<D, DB>(acc, p.scale, p.dQ + ((size_t)row * p.Hq + head) * D, half);
    } else {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) aq[(db * 16 + r) * 64 + lane] = acc[db][r];
    }
}

// ---------------------------------------------------------------------------------------
// Row statistics in the form the dK/dV kernel consumes, so that its steps can fetch them with a
// plain 256-byte copy: out[head][32-row block][0..31] = LSE * log2(e), [32..63] = -Delta.
__global__ __launch_bounds__(256) void stat_pack_kernel(const float* __restrict__ LSE, const float* __restrict__ Delta,
                                                        int64_t stride, int64_t n_blocks, int Hq,
                                                        int64_t out_head_stride_blocks, float* __restrict__ out)
{
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (head, block) pair
    if (item >= n_blocks * Hq) return;
    const int64_t head = item / n_blocks, blk = item % n_blocks;
    const int t = threadIdx.x & 63;
    const float v = (t < 32 ? LSE : Delta - 32)[(size_t)head * stride + blk * 32 + t];
    out[((size_t)head * out_head_stride_blocks + blk) * 64 + t] = t < 32 ? v * LOG2E : -v;
}

// ---------------------------------------------------------------------------------------
// Delta[h][row] = sum_d dO * O.  One wave per (row, head) pair group: lanes split channels.
template <typename T>
__device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<uint16_t>(const uint16_t* p)
{
    return __uint_as_float(((unsigned)*p) << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void delta_kernel(const T* __restrict__ O, const T* __restrict__ dO,
                                                    int64_t rows, int Hq, int D, float* __restrict__ Delta,
                                                    int64_t stride)
{
    // 16 lanes per (row, head): 4 pairs per wave, 16 pairs per workgroup
    const int tid = threadIdx.x;
    const int64_t pair = (int64_t)blockIdx.x * 16 + (tid >> 4);
    const int sub = tid & 15;
    if (pair >= rows * Hq) return;  // whole 16-lane groups leave together
    const T* o = O + (size_t)pair * D;
    const T* g = dO + (size_t)pair * D;
    float acc = 0.f;
    for (int d = sub; d < D; d += 16) acc += ld<T>(o + d) * ld<T>(g + d);
#pragma unroll
    for (int m = 8; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (sub == 0) {
        const int64_t row = pair / Hq;
        const int h = (int)(pair % Hq);
        Delta[(size_t)h * stride + row] = acc;
    }
}


// Exact Delta for the first rows of the sequence: Delta_i = sum_j p_ij (dO_i . v_j).
// rowsum(dO * O) inherits the bf16 rounding of the stored O; for a row with only a few keys
// the softmax is often peaked, dS = p (dP - Delta) then cancels almost completely and that
// rounding dominates dQ.  Its weight decays like 1/sqrt(row), so only the head of the
// sequence is recomputed (plain FMA, one wave per (row, head); the cost is negligible).
__global__ __launch_bounds__(256) void delta_head_kernel(const uint16_t* __restrict__ Q,
                                                         const uint16_t* __restrict__ dO,
                                                         const uint16_t* __restrict__ K,
                                                         const uint16_t* __restrict__ V,
                                                         const float* __restrict__ LSE, int64_t stat_stride,
                                                         int rows, int Hq, int Hkv, int D, float scale,
                                                         float* __restrict__ Delta)
{
    const int lane = threadIdx.x & 63;
    const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= rows * Hq) return;  // wave-uniform
    const int row = pair / Hq, head = pair % Hq;
    const int kvh = head / (Hq / Hkv);
    const uint16_t* q = Q + ((size_t)row * Hq + head) * D;
    const uint16_t* go = dO + ((size_t)row * Hq + head) * D;
    const float lse = LSE[(size_t)head * stat_stride + row];
    float acc = 0.f;
    for (int j = lane; j <= row; j += 64) {
        const uint16_t* k = K + ((size_t)j * Hkv + kvh) * D;
        const uint16_t* v = V + ((size_t)j * Hkv + kvh) * D;
        float s = 0.f, dp = 0.f;
        for (int d = 0; d < D; ++d) {
            s = fmaf(ld<uint16_t>(q + d), ld<uint16_t>(k + d), s);
            dp = fmaf(ld<uint16_t>(go + d), ld<uint16_t>(v + d), dp);
        }
        acc = fmaf(expf(scale * s - lse), dp, acc);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (lane == 0) Delta[(size_t)head * stat_stride + row] = acc;
}

}  // namespace

int bwd_k_tile(int D) { (void)D; return NWAVE * 32; }
int bwd_q_tile(int D) { (void)D; return NWAVE * 32; }
size_t bwd_acc_dq_bytes(int64_t n_q, int Hq, int D) { return (size_t)n_q * Hq * dpad(D) * sizeof(float); }
size_t bwd_acc_dkv_bytes(int64_t n_k, int Hkv, int D) { return (size_t)n_k * Hkv * dpad(D) * sizeof(float); }

static BwdKernelArgs to_kernel_args(const BwdArgs& a)
{
    BwdKernelArgs k;
    k.Q = (const uint16_t*)a.Q; k.dO = (const uint16_t*)a.dO;
    k.K = (const uint16_t*)a.K; k.V = (const uint16_t*)a.V;
    k.Qnat = (const u32x4*)a.Qnat;
    k.dOnat = (const u32x4*)a.dOnat;
    k.q_head_stride_blocks = a.q_head_stride_blocks;
    k.Knat = (const u32x4*)a.Knat; k.Vnat = (const u32x4*)a.Vnat;
    k.kv_head_stride_blocks = a.kv_head_stride_blocks;
    k.LSE = a.LSE; k.Delta = a.Delta; k.row_stat_stride = a.row_stat_stride;
    k.stat2 = a.stat2;
    k.q_pos0 = a.q_pos0; k.k_pos0 = a.k_pos0;
    k.n_q = (int)a.n_q; k.n_k = (int)a.n_k;
    k.Hq = a.Hq; k.Hkv = a.Hkv; k.g = a.Hq / a.Hkv; k.flags = a.flags;
    k.scale = a.scale; k.c = a.scale * LOG2E;
    k.acc_dq = a.acc_dq; k.acc_dk = a.acc_dk; k.acc_dv = a.acc_dv;
    k.dQ = (uint16_t*)a.dQ; k.dK = (uint16_t*)a.dK; k.dV = (uint16_t*)a.dV;
    k.dS = (u32x4*)a.dS_frag;
    return k;
}

void launch_bwd_dkdv(const BwdArgs& a, hipStream_t st)
{
    const BwdKernelArgs k = to_kernel_args(a);
    dim3 grid((unsigned)((a.n_k / bwd_k_tile(a.D)) * a.Hkv));
    // (dS fragment pairs are indexed in 32 bits inside the kernels; the API layer sizes the buffer)
    if (a.dS_frag) {
        if (a.D == 128) bwd_dkdv_kernel_w4<128, true><<<grid, 256, 0, st>>>(k);
        else if (a.D == 80) bwd_dkdv_kernel_w4<80, true><<<grid, 256, 0, st>>>(k);
        else bwd_dkdv_kernel_w4<64, true><<<grid, 256, 0, st>>>(k);
        return;
    }
    if (a.D == 128) bwd_dkdv_kernel_w4<128, false><<<grid, 256, 0, st>>>(k);
    else if (a.D == 80) bwd_dkdv_kernel_w4<80, false><<<grid, 256, 0, st>>>(k);
    else bwd_dkdv_kernel_w4<64, false><<<grid, 256, 0, st>>>(k);
}

// dQ of the launch from the dS fragments that launch_bwd_dkdv wrote for the same ranges
void launch_bwd_dq_from_ds(const BwdArgs& a, hipStream_t st)
{
    const BwdKernelArgs k = to_kernel_args(a);
    dim3 grid((unsigned)((a.n_q / bwd_q_tile(a.D)) * a.Hq));
    if (a.D == 128) bwd_dq_ds_kernel<128><<<grid, NTHREAD, 0, st>>>(k);
    else if (a.D == 80) bwd_dq_ds_kernel<80><<<grid, NTHREAD, 0, st>>>(k);
    else bwd_dq_ds_kernel<64><<<grid, NTHREAD, 0, st>>>(k);
}

void launch_bwd_dq(const BwdArgs& a, hipStream_t st)
{
    const BwdKernelArgs k = to_kernel_args(a);
    dim3 grid((unsigned)((a.n_q / bwd_q_tile(a.D)) * a.Hq));
    if (a.D == 128) bwd_dq_kernel<128><<<grid, NTHREAD, 0, st>>>(k);
    else if (a.D == 80) bwd_dq_kernel<80><<<grid, NTHREAD, 0, st>>>(k);
    else bwd_dq_kernel<64><<<grid, NTHREAD, 0, st>>>(k);
}

void launch_stat_pack(const float* LSE, const float* Delta, int64_t stride, int64_t rows, int Hq,
                      int64_t out_head_stride_blocks, float* out, hipStream_t st)
{
    const int64_t items = rows / 32 * Hq;
    if (items <= 0) return;
    stat_pack_kernel<<<dim3((unsigned)((items + 3) / 4)), 256, 0, st>>>(LSE, Delta, stride, rows / 32, Hq,
                                                                       out_head_stride_blocks, out);
}

void launch_delta(const void* O, const void* dO, int64_t rows, int Hq, int D, int is_bf16,
                  float* Delta, int64_t delta_stride, hipStream_t st)
{
    const int64_t pairs = rows * Hq;
    dim3 grid((unsigned)((pairs + 15) / 16));
    if (is_bf16)
        delta_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)O, (const uint16_t*)dO, rows, Hq, D, Delta, delta_stride);
    else
        delta_kernel<float><<<grid, 256, 0, st>>>((const float*)O, (const float*)dO, rows, Hq, D, Delta, delta_stride);
}

void launch_delta_head(const void* Q, const void* dO, const void* K, const void* V, const float* LSE,
                       int64_t stat_stride, int rows, int Hq, int Hkv, int D, float scale, float* Delta,
                       hipStream_t st)
{
    dim3 grid((unsigned)((rows * Hq + 3) / 4));
    delta_head_kernel<<<grid, 256, 0, st>>>((const uint16_t*)Q, (const uint16_t*)dO, (const uint16_t*)K,
                                            (const uint16_t*)V, LSE, stat_stride, rows, Hq, Hkv, D, scale,
                                            Delta);
}

}  // namespace fpdt
