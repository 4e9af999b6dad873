// Internal declarations shared by the translation units of libfpdt.so.
// Host-side launch wrappers: each validates nothing (the API layer does) and
// only enqueues kernels on the given stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fpdt {

typedef uint16_t bf16_bits;  // storage type of a bfloat16 element on the host side

// ---------------------------------------------------------------------------
// MFMA fragment packing (bf16).  Rows come in blocks of 32; 1 KiB "fragments"
// hold 64 lanes x 8 bf16 in the exact order a v_mfma_f32_32x32x16_bf16 operand
// wants them, so the hot kernels stream them global -> LDS -> register with no
// shuffling.
//   NAT (contraction over channels):  [head][row_block][t = D/16][lane][8]
//       lane (r = lane%32, h = lane/32) holds X[row0 + r][16t + 8h + e]
//   TR  (contraction over rows):      [head][row_block][s = 2][db = DP/32][lane][8]
//       lane (c = lane%32, h = lane/32) holds X[row0 + 8(2s + e/4) + 4h + e%4][32db + c]
//       (zero where 32db + c >= D); the row order matches the accumulator
//       layout of a 32x32 MFMA result, so a register-resident score tile can be
//       the other operand directly.
// ---------------------------------------------------------------------------
static inline int dpad(int D) { return (D + 31) / 32 * 32; }
static inline size_t nat_block_bytes(int D) { return (size_t)(D / 16) * 1024; }
static inline size_t tr_block_bytes(int D) { return (size_t)(2 * (dpad(D) / 32)) * 1024; }

// Pack `rows` rows (multiple of 32) of X [rows, H, D] into NAT and/or TR form.
// Output head stride is given in 32-row blocks (>= rows/32) so that a chunk
// can be packed into its slot of a whole-sequence buffer.
void launch_pack(const void* X, int64_t rows, int H, int D, void* nat, void* tr,
                 int64_t head_stride_blocks, hipStream_t st);

// ---------------------------------------------------------------------------
// bf16 forward sweep: query rows [q_pos0, q_pos0 + n_q) against keys
// [k_pos0, k_pos0 + n_keys) (causal: key position <= query position).
// ---------------------------------------------------------------------------
enum { SWEEP_INIT = 1, SWEEP_FINAL = 2 };

struct FwdArgs {
    const void* Q;      // first query row of the launch, [n_q, Hq, D] bf16
    const void* Knat;   // packed NAT, block 0 = keys k_pos0..k_pos0+31
    const void* Vtr;    // packed TR
    int64_t kv_head_stride_blocks;
    void* O;            // [n_q, Hq, D] bf16 (written when SWEEP_FINAL)
    float* LSE;         // &LSE[0][q_pos0]; head stride lse_stride
    int64_t lse_stride;
    float* st_acc;      // carried un-normalised output, fragment order
    float* st_ml;       // carried running max / sum
    int64_t q_pos0, k_pos0;
    int64_t n_q, n_keys;
    int Hq, Hkv, D;
    float scale;
    int flags;          // SWEEP_INIT: start from empty state; SWEEP_FINAL: normalise + write O, LSE
};
int fwd_q_tile(int D);                                    // query rows per workgroup
size_t fwd_state_acc_bytes(int64_t n_q, int Hq, int D);   // carried state for n_q rows
size_t fwd_state_ml_bytes(int64_t n_q, int Hq, int D);
void launch_fwd_sweep(const FwdArgs& a, hipStream_t st);

// ---------------------------------------------------------------------------
// bf16 backward
// ---------------------------------------------------------------------------
// Delta[h][row] = sum_d dO[row,h,d] * O[row,h,d].
void launch_delta(const void* O, const void* dO, int64_t rows, int Hq, int D, int is_bf16,
                  float* Delta, int64_t delta_stride, hipStream_t st);

// Overwrite Delta for rows [0, rows) of the sequence with sum_j p_ij (dO_i . v_j), which does
// not depend on the rounded O.  All pointers are at row 0; rows <= DELTA_HEAD_ROWS.
enum { DELTA_HEAD_ROWS = 256 };
void launch_delta_head(const void* Q, const void* dO, const void* K, const void* V, const float* LSE,
                       int64_t stat_stride, int rows, int Hq, int Hkv, int D, float scale, float* Delta,
                       hipStream_t st);

// out[head][block][64] = 32 x LSE * log2(e), 32 x -Delta for `rows` query rows (multiple of 32)
void launch_stat_pack(const float* LSE, const float* Delta, int64_t stride, int64_t rows, int Hq,
                      int64_t out_head_stride_blocks, float* out, hipStream_t st);

enum { ACC_LOAD = 1, ACC_FINAL = 2 };

struct BwdArgs {
    // raw tensors at the first row of the launch's ranges
    const void* Q;   // [n_q, Hq, D]
    const void* dO;  // [n_q, Hq, D]
    const void* K;   // [n_k, Hkv, D]
    const void* V;   // [n_k, Hkv, D]
    // packed forms of the same ranges
    const void* Qnat; const void* dOnat;
    int64_t q_head_stride_blocks;
    const void* Knat; const void* Vnat;
    int64_t kv_head_stride_blocks;
    const float* LSE;    // &LSE[0][q_pos0], head stride row_stat_stride (natural log)
    const float* Delta;  // &Delta[0][q_pos0], same stride
    int64_t row_stat_stride;
    // the same statistics as the dK/dV kernel consumes them (launch_stat_pack), block 0 = rows
    // q_pos0 .. q_pos0 + 31, head stride q_head_stride_blocks blocks of 64 floats
    const float* stat2 = nullptr;
    int64_t q_pos0, k_pos0, n_q, n_k;
    int Hq, Hkv, D;
    float scale;
    // accumulators (fp32, fragment order, one slot per workgroup of the launch)
    float* acc_dq;   // dQ kernel
    float* acc_dk;   // dK/dV kernel
    float* acc_dv;
    void* dQ;        // [n_q, Hq, D] bf16, written when flags has ACC_FINAL
    void* dK;        // [n_k, Hkv, D] bf16
    void* dV;
    int flags;       // ACC_LOAD: start from the accumulators; ACC_FINAL: round + write outputs
    // stored-dS backward: n_q * n_k * Hq bf16 of dS tiles, written by the dK/dV kernel of the
    // launch and read by launch_bwd_dq_from_ds; null = dQ recomputes S and dP (launch_bwd_dq)
    void* dS_frag = nullptr;
};
size_t bwd_acc_dq_bytes(int64_t n_q, int Hq, int D);
size_t bwd_acc_dkv_bytes(int64_t n_k, int Hkv, int D);  // each of dK, dV
int bwd_k_tile(int D);
int bwd_q_tile(int D);
void launch_bwd_dkdv(const BwdArgs& a, hipStream_t st);
void launch_bwd_dq(const BwdArgs& a, hipStream_t st);
void launch_bwd_dq_from_ds(const BwdArgs& a, hipStream_t st);
static inline size_t bwd_ds_bytes(int64_t n_q, int64_t n_k, int Hq) { return (size_t)n_q * (size_t)n_k * Hq * 2; }

// ---------------------------------------------------------------------------
// fp32 path (accuracy path; plain FMA, one wave per row)
// ---------------------------------------------------------------------------
struct F32FwdArgs {
    const float* Q; const float* K; const float* V;  // at first row of the ranges
    float* O; float* LSE; int64_t lse_stride;
    float* st_acc; float* st_ml;  // [n_q, Hq, D], [n_q, Hq, 2]
    int64_t q_pos0, k_pos0, n_q, n_k;
    int Hq, Hkv, D;
    float scale;
    int flags;  // SWEEP_INIT / SWEEP_FINAL
};
void launch_f32_fwd_pair(const F32FwdArgs& a, hipStream_t st);

struct F32BwdArgs {
    const float* Q; const float* dO; const float* K; const float* V;
    const float* LSE; const float* Delta; int64_t row_stat_stride;
    float* dQ; float* dK; float* dV;  // accumulated in place (caller zero-fills first)
    int64_t q_pos0, k_pos0, n_q, n_k;
    int Hq, Hkv, D;
    float scale;
};
void launch_f32_bwd_pair(const F32BwdArgs& a, hipStream_t st);

// merge of two partial results (both dtypes)
void launch_merge(const void* Oa, const float* La, const void* Ob, const float* Lb, void* Oo,
                  float* Lo, int64_t rows, int Hq, int D, int is_bf16, hipStream_t st);

// Calibration loops (csrc/calibrate.hip): returns the waves per SIMD of the launched variant, 0 for
// an unknown kind.  One launch executes blocks * (waves per SIMD * 4) * iters * 24 MFMAs.
enum { CALIBRATE_MFMA_PER_TRIP = 24 };
void launch_calibrate_fill(void* in, hipStream_t st);
int launch_calibrate(int kind, float* out, const void* in, int iters, int blocks, hipStream_t st);

// zero-fill by kernel (safe under graph capture)
void launch_zero(void* p, size_t bytes, hipStream_t st);
void launch_fill_bytes(void* p, size_t bytes, unsigned char byte, hipStream_t st);

}  // namespace fpdt
