/*
 * fpdt.h -- C ABI of the MI355X chunked causal attention library (libfpdt.so).
 *
 * One GPU's head share of the paper's sequence-chunked distributed attention
 * (Sec. 4.1 forward, Sec. 4.2 backward): the sequence of S tokens is cut into
 * u = S / chunk chunks; query chunk m attends the key/value chunks i <= m one
 * chunk pair at a time with online-softmax accumulation, the causal mask is
 * applied on diagonal pairs only, and key/value chunks that are not in use may
 * live in pinned host memory and are prefetched back through a double buffer
 * while earlier pairs compute (Sec. 4.2, double buffering).  The result is
 * ordinary causal softmax attention, O = softmax(scale * Q K^T) V, and its
 * gradients.
 *
 * Conventions common to every entry point
 *   - batch 1; tensors are row-major contiguous [S, H, D] ("token, head,
 *     channel"), so that one chunk of a tensor is one contiguous slab;
 *     Q, O, dO, dQ have Hq heads, K, V, dK, dV have Hkv heads; query head h
 *     reads KV head h / (Hq / Hkv) (grouped-query attention) and the gradient
 *     of a KV head is the sum over its query heads.
 *   - LSE is the natural-log log-sum-exp of the scaled scores, fp32, [Hq, S].
 *   - dtype FPDT_DTYPE_BF16: tensors are bfloat16, arithmetic is bf16 MFMA with
 *     fp32 accumulation; FPDT_DTYPE_F32: tensors and arithmetic are fp32.
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers must be pinned (hipHostMalloc) memory.  The caller owns every
 *     buffer.  The library allocates no device memory; it lazily creates one
 *     side stream and a few events per process for the offload pipeline.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work: everything is ordered after prior work on
 *     `stream` and is complete when `stream` is.  Buffers (host ones included)
 *     must stay valid and untouched until then.
 *   - Every function returns an fpdt_status; nothing throws or aborts.  On any
 *     error other than FPDT_ERR_HIP nothing has been enqueued.  Text for the
 *     last error of the calling thread: fpdt_last_error().
 */
#ifndef FPDT_H
#define FPDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FPDT_OK = 0,
    FPDT_ERR_INVALID_ARG = 1, /* null pointer, S<=0, chunk<=0, S % chunk != 0, Hq % Hkv != 0,
                                 scale not finite or <= 0, unknown dtype or flag bits, both
                                 loop-order flags                                            */
    FPDT_ERR_UNSUPPORTED = 2, /* D not in {64, 80, 128}; bf16 chunk not a multiple of
                                 FPDT_CHUNK_MULTIPLE; fp32 with offload flags; sizes beyond
                                 the 32-bit launch limits                                    */
    FPDT_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned (256 B) or too small             */
    FPDT_ERR_HIP = 4          /* a HIP runtime call failed; see fpdt_last_error()            */
} fpdt_status;

enum { FPDT_DTYPE_F32 = 0, FPDT_DTYPE_BF16 = 1 };

/* chunk (and therefore S) must be a multiple of this for bf16; fp32 accepts any chunk. */
enum { FPDT_CHUNK_MULTIPLE = 256 };

enum {
    /* K, V (forward and backward) and dK, dV (backward) are pinned HOST pointers; the
     * library keeps at most two key/value chunks on the device (Sec. 4.1: only the
     * chunks in use are in HBM; Sec. 4.2: double buffer).                              */
    FPDT_KV_ON_HOST = 1u << 0,
    /* Q, O, dO, dQ and LSE are pinned HOST pointers as well (forward: Q in, O and LSE
     * out; backward: Q, O, dO, LSE in, dQ out) and are streamed chunk by chunk
     * (Sec. 4.1: q, k, v chunks are offloaded once the forward is done with them).     */
    FPDT_ACT_ON_HOST = 1u << 1,
    /* Backward chunk-pair loop order (Sec. 4.2).  KV_OUTER is the paper's: outer loop
     * over key/value chunks j, inner over query chunks i >= j.  Q_OUTER: outer over
     * query chunks i, inner over j <= i.  Neither bit: the library picks
     * (KV_OUTER unless FPDT_ACT_ON_HOST is set; FPDT_ACT_ON_HOST with KV_OUTER is
     * FPDT_ERR_UNSUPPORTED).                                                           */
    FPDT_BWD_KV_OUTER = 1u << 2,
    FPDT_BWD_Q_OUTER = 1u << 3,
    /* Run the chunk-pair schedule launch by launch (carried fp32 state between pairs)
     * even when every tensor is resident.  Without this bit and without offload flags
     * the bf16 path ignores `chunk` (beyond validating it) and runs ONE causal sweep over
     * the whole sequence per kernel: the same set of (query, key) tiles, no carried state
     * between launches.  The offload pipeline always runs pair by pair, with the same
     * kernels in the same order as this mode: the two agree bit for bit.  fp32 always
     * runs pair by pair.                                                               */
    FPDT_PAIRWISE = 1u << 4,
    /* Backward only (bf16; the forward ignores it): the stored-dS backward.  The paper's
     * backward, like any FlashAttention backward, recomputes the probabilities per chunk
     * pair (Sec. 3.1, 4.2); the two-kernel form used here (no atomics) recomputes the
     * scores and dP twice, once for dK/dV and once for dQ: 7 GEMMs per pair for the
     * algorithmic 5.  With this flag the dK/dV kernel also writes the rounded dS tiles of
     * the pair (the very bf16 values its own MFMAs consume) to the workspace, and dQ is
     * one GEMM over them: 5 executed GEMMs, the same dQ numerics (dS was already rounded
     * to bf16 for its MFMA), for chunk * chunk * Hq * 2 bytes of workspace (64 GiB at
     * chunk = 65,536 and Hq = 8: sized for a 288 GB GPU) and that many bytes of HBM traffic
     * each way per pair.  Implies the pair-by-pair schedule (as FPDT_PAIRWISE).           */
    FPDT_BWD_STORE_DS = 1u << 5
};

/*
 * Bytes of device workspace fpdt_attn_fwd (is_bwd = 0) or fpdt_attn_bwd (is_bwd = 1)
 * needs for these arguments; 0 if the arguments are invalid or unsupported (call the
 * entry point itself for the status).  With FPDT_KV_ON_HOST the forward workspace
 * holds two key/value chunk buffers plus per-chunk state: it does not grow with S.
 * The backward workspace under the offload flags is chunk-sized buffers (packed operands, raw
 * and output staging, the accumulators of the side the outer loop holds fixed) PLUS state
 * that grows with S, because the gradient of the side the inner loop walks is accumulated in
 * fp32 on the device from one outer iteration to the next:
 *   KV-outer (default with FPDT_KV_ON_HOST alone): dQ accumulator S * Hq * dpad(D) * 4 bytes
 *       and Delta S * Hq * 4 (8 GiB + 64 MiB at S = 2M, Hq = 8, D = 128);
 *   Q-outer: dK and dV accumulators 2 * S * Hkv * dpad(D) * 4 bytes (2 GiB at S = 2M,
 *       Hkv = 2), plus Delta S * Hq * 4 unless FPDT_ACT_ON_HOST streams it per chunk;
 * dpad(D) = D rounded up to a multiple of 32.
 */
size_t fpdt_attn_workspace_bytes(int64_t S, int64_t chunk, int Hq, int Hkv, int D, int dtype,
                                 unsigned flags, int is_bwd);

/*
 * Chunk size to use for a sequence of S tokens (Sec. 5.3: a chunk that is too small starves
 * the GPU, one that is too large wastes device memory on chunk buffers; the paper settles on
 * 64K tokens).  Returns the largest chunk c <= FPDT_PREFERRED_CHUNK with S % c == 0, c a
 * multiple of FPDT_CHUNK_MULTIPLE (bf16 only), for which both workspaces
 * (fpdt_attn_workspace_bytes with is_bwd = 0 and 1) fit in max_workspace_bytes (0 = no
 * limit).  Why that cap: one launch of the dK/dV kernel has chunk / 256 * Hkv workgroups,
 * which fills the 256 compute units only from 32K tokens on at two KV heads, and every
 * chunk pair costs a fixed launch, state load and state store; measured on the Llama-8B head
 * share with K/V offloaded the throughput rises steeply up to 32K tokens, by 3% (S = 256K)
 * or 1% (S = 2M) from 32K to 64K, and by 0.3% at most from 64K to 128K, while every chunk-sized
 * buffer doubles.  64K is the knee of that curve on this machine as well.
 * Returns 0 when the arguments are invalid or no chunk fits (fpdt_last_error says which).
 * Host logic only: no device is touched.
 */
enum { FPDT_PREFERRED_CHUNK = 65536 };
int64_t fpdt_attn_pick_chunk(int64_t S, int Hq, int Hkv, int D, int dtype, unsigned flags,
                             size_t max_workspace_bytes);

/*
 * Forward (Sec. 4.1, Figs. 4-5).  For every query chunk m = 0..u-1, fold in the
 * key/value chunks i = 0..m (earlier chunks first, the masked diagonal pair last),
 * carrying the running row maximum, row sum and un-normalised output in fp32, and
 * normalise once at the end of the chunk.
 *   Q [S,Hq,D], K, V [S,Hkv,D]  in   (device; host per the flags)
 *   O [S,Hq,D], LSE [Hq,S] fp32 out  (device; host with FPDT_ACT_ON_HOST)
 *   workspace: device memory, 256-byte aligned, >= fpdt_attn_workspace_bytes(..., 0)
 * Stream capture: forward and backward only enqueue kernels, copies and event waits (the
 * offload schedules fork onto the library's side streams and join back through events), so
 * they may be captured in a HIP graph; the tensors and the workspace, host buffers included,
 * must then stay valid for every replay.
 */
int fpdt_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE, int64_t S,
                  int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype, unsigned flags,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * fpdt_attn_fwd for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as fpdt_attn_fwd
 * (same kernels, so the same bits), except that the workspace is a device array built into the
 * library, FPDT_NOALLOC_SCRATCH_BYTES per GPU, held from the library's load until the process
 * ends.  The call makes no hipMalloc / hipFree, creates no stream or event and records no
 * profiling events (fpdt_profile_enable does not see it).
 *   - Tensors are resident: FPDT_KV_ON_HOST / FPDT_ACT_ON_HOST give FPDT_ERR_UNSUPPORTED.
 *   - Sizes whose fpdt_attn_workspace_bytes(..., 0) exceeds FPDT_NOALLOC_SCRATCH_BYTES give
 *     FPDT_ERR_WORKSPACE and enqueue nothing.  bf16 without FPDT_PAIRWISE needs
 *     S / 32 * Hkv * (D / 16 + 2 * ceil(D / 32)) KiB: S * Hkv <= 65,536 at D = 128.
 *   - Every call on a GPU uses that GPU's one array and finds the previous call's contents in
 *     it.  Nothing has to start at zero (a call writes every byte it later reads), but two
 *     calls that overlap in time on one GPU (different streams, or different threads) race on
 *     it: keep such calls on one stream, or order them with events.
 *   - The array's address is looked up on the first call on each device (hipGetSymbolAddress;
 *     not a stream operation): make that first call outside stream capture.
 */
enum { FPDT_NOALLOC_SCRATCH_BYTES = 32 << 20 };
int fpdt_attn_fwd_noalloc(const void *Q, const void *K, const void *V, void *O, float *LSE,
                          int64_t S, int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype,
                          unsigned flags, void *stream);

/*
 * Backward (Sec. 4.2, Fig. 7; operand set of Sec. 3.1).  Computes
 * Delta = rowsum(dO * O) once, then for every chunk pair (i >= j), in the chosen loop
 * order, recomputes p = exp(scale q k^T - LSE) (masked on diagonal pairs) and adds
 * the pair's share to dQ_i, dK_j, dV_j in fp32; gradients are rounded to the tensor
 * dtype once a chunk's accumulation is complete.
 *   Q, O, dO [S,Hq,D], K, V [S,Hkv,D], LSE [Hq,S]  in   (O, LSE as written by the forward)
 *   dQ [S,Hq,D], dK, dV [S,Hkv,D]                  out  (fully overwritten)
 *   workspace: device memory, 256-byte aligned, >= fpdt_attn_workspace_bytes(..., 1)
 */
int fpdt_attn_bwd(const void *Q, const void *K, const void *V, const void *O, const float *LSE,
                  const void *dO, void *dQ, void *dK, void *dV, int64_t S, int64_t chunk, int Hq,
                  int Hkv, int D, float scale, int dtype, unsigned flags, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * Block-sparse variants (Sec. 5.5: with block-sparse attention only part of the key/value
 * chunks is fetched from host memory, the queries are always the whole sequence).
 * chunk_mask: u x u bytes in HOST memory (u = S / chunk), row = query chunk m, column = key
 * chunk i; query chunk m attends key chunk i iff i <= m and chunk_mask[m * u + i] != 0
 * (entries with i > m are ignored).  Pairs that are switched off are neither fetched nor
 * computed; inside the pairs that are kept the arithmetic is that of fpdt_attn_fwd /
 * fpdt_attn_bwd, so an all-ones mask gives the same bits as those with FPDT_PAIRWISE.
 * The mask is read before the call returns.  Every diagonal entry must be set (a query row
 * always keeps its own key): FPDT_ERR_INVALID_ARG otherwise.  The schedule is pair by pair:
 * size the workspace with fpdt_attn_workspace_bytes(..., flags | FPDT_PAIRWISE, ...).
 * All other arguments, layouts and errors as in fpdt_attn_fwd / fpdt_attn_bwd; the backward
 * must be given the same mask as the forward that produced O and LSE.
 */
int fpdt_attn_fwd_blocksparse(const void *Q, const void *K, const void *V, void *O, float *LSE,
                              int64_t S, int64_t chunk, int Hq, int Hkv, int D, float scale,
                              int dtype, unsigned flags, const unsigned char *chunk_mask,
                              void *workspace, size_t workspace_bytes, void *stream);
int fpdt_attn_bwd_blocksparse(const void *Q, const void *K, const void *V, const void *O,
                              const float *LSE, const void *dO, void *dQ, void *dK, void *dV,
                              int64_t S, int64_t chunk, int Hq, int Hkv, int D, float scale,
                              int dtype, unsigned flags, const unsigned char *chunk_mask,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Online-softmax merge of two partial attention results over disjoint key sets
 * (the rescale of an intermediate result when a further chunk is folded in,
 * Sec. 4.1): LSE = logaddexp(LSE_a, LSE_b),
 * O = O_a exp(LSE_a - LSE) + O_b exp(LSE_b - LSE).
 *   O_a, O_b, O_out [rows,Hq,D] (dtype), LSE_a, LSE_b, LSE_out [Hq,rows] fp32, all
 *   device; O_out / LSE_out may alias either input.  A partial with LSE = -inf
 *   (no keys seen) contributes nothing.
 */
int fpdt_attn_merge(const void *O_a, const float *LSE_a, const void *O_b, const float *LSE_b,
                    void *O_out, float *LSE_out, int64_t rows, int Hq, int D, int dtype,
                    void *stream);

/*
 * Host-link traffic of the calling thread's most recent fpdt_attn_fwd / fpdt_attn_bwd
 * call: bytes enqueued host-to-device and device-to-host (0, 0 without offload flags).
 * Either pointer may be NULL.
 */
int fpdt_last_link_bytes(uint64_t *h2d_bytes, uint64_t *d2h_bytes);

/*
 * Kernel and copy timing for benchmarks.  While enabled, every launch of the three MFMA
 * kernels (forward sweep; backward dK/dV; backward dQ) and every host-link copy the
 * library enqueues is bracketed by HIP events on the stream it runs on.
 * fpdt_profile_read waits for the recorded events of one kind, returns the summed
 * duration in milliseconds and the number of launches, and forgets them.
 */
enum { FPDT_PROF_FWD = 0, FPDT_PROF_DKDV = 1, FPDT_PROF_DQ = 2, FPDT_PROF_H2D = 3,
       FPDT_PROF_D2H = 4, FPDT_PROF_KINDS = 5 };
int fpdt_profile_enable(int on);
int fpdt_profile_read(int kind, double *total_ms, int64_t *launches);

/*
 * Calibration of the roofline the attention kernels are measured against (Sec. 5.2 reports
 * model FLOPs utilisation against the hardware's peak): what this GPU sustains on the MFMA
 * instruction of the kernels (32x32x16 bf16, fp32 accumulation) with random operands of
 * order one -- its clock under load depends on the data -- alone and in the company the
 * attention kernels keep.  One workgroup per compute unit runs a fixed number of trips of a
 * register / LDS loop; nothing on the attention path calls this.
 *   kind  FPDT_CAL_MFMA_REG_2W / _1W      MFMAs on register operands, two / one wave per SIMD
 *         FPDT_CAL_SOFTMAX_REG_2W / _1W   the same with the forward's softmax instructions
 *                                         between the MFMAs: per MFMA one multiply-add, one
 *                                         exp2, one add and a packed bf16 conversion or a
 *                                         three-way maximum
 *         FPDT_CAL_MFMA_LDS1_2W           the A operand of every MFMA freshly read from LDS
 *                                         (1 KiB per MFMA: the forward and the dQ kernel)
 *         FPDT_CAL_MFMA_LDS2_1W           one LDS fragment per two MFMAs, one wave per SIMD
 *                                         (the dK/dV kernel)
 *         FPDT_CAL_SOFTMAX_LDS1_2W, FPDT_CAL_SOFTMAX_LDS2_1W   both together
 *   iters      trips of 24 MFMAs per wave (20000 runs about 0.1 s)
 *   workspace  device memory, 256-byte aligned, >= FPDT_CAL_WORKSPACE_BYTES
 *   tflops     out: executed MFMA TFLOP/s over the whole GPU;  ms: out (may be NULL)
 * Synchronous: returns when the run has finished on `stream`.
 */
enum { FPDT_CAL_MFMA_REG_2W = 0, FPDT_CAL_MFMA_REG_1W = 1, FPDT_CAL_SOFTMAX_REG_2W = 2,
       FPDT_CAL_SOFTMAX_REG_1W = 3, FPDT_CAL_MFMA_LDS1_2W = 4, FPDT_CAL_MFMA_LDS2_1W = 5,
       FPDT_CAL_SOFTMAX_LDS1_2W = 6, FPDT_CAL_SOFTMAX_LDS2_1W = 7, FPDT_CAL_KINDS = 8 };
enum { FPDT_CAL_WORKSPACE_BYTES = 1 << 20 };
int fpdt_calibrate_mfma(int kind, int iters, void *workspace, size_t workspace_bytes,
                        double *tflops, double *ms, void *stream);

/*
 * Event-ordering checks for the offload pipeline (Sec. 4.2: copies on side streams, one buffer
 * being filled while the other is used).  For tests of the pipeline itself, not for production:
 *   FPDT_DEBUG_POISON_STAGING  every device staging buffer is filled with 0xFF bytes (NaNs)
 *                              right before the host-to-device copy into it, on the copy's
 *                              stream: a kernel that does not wait for the copy reads NaNs;
 *   FPDT_DEBUG_DELAY_COPIES    a 48 MiB dummy copy is queued in front of every staged copy
 *                              (either direction), so copies finish much later than they are
 *                              enqueued: a missing wait shows up as stale or poisoned data,
 *                              a missing buffer-release wait as a late overwrite.
 * With either flag a correct pipeline still returns bit for bit what the resident run returns.
 * flags = 0 switches both off.  The first call with FPDT_DEBUG_DELAY_COPIES allocates the dummy
 * buffers (48 MiB pinned host + 48 MiB device per GPU, kept until the process ends).
 */
enum { FPDT_DEBUG_POISON_STAGING = 1u << 0, FPDT_DEBUG_DELAY_COPIES = 1u << 1 };
int fpdt_debug_configure(unsigned flags);

/* Text describing the calling thread's most recent error ("" if none). Never NULL. */
const char *fpdt_last_error(void);

/* Library version string, e.g. "fpdt 0.1 gfx950". */
const char *fpdt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FPDT_H */
