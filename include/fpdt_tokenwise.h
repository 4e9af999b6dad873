/*
 * fpdt_tokenwise.h -- C ABI of the token-wise chunked neighbours of the attention path
 * (Sec. 5.4, "Chunk Granularity"): operations whose cost is linear in the sequence length and
 * whose intermediate buffers, not their FLOPs, are the problem at long sequences.  They are
 * chunked along the sequence without offloading; the intermediates exist for one chunk at a
 * time.
 *
 *   fpdt_tw_loss_fwd_bwd   softmax cross-entropy over the vocabulary with its last linear
 *                          projection, forward and backward fused per chunk: the fp32 logits
 *                          [rows, vocab] never exist for more than one chunk (Sec. 5.4 names
 *                          the loss over a large vocabulary as the place where memory peaks
 *                          and suggests vocab / hidden * 2 chunks).
 *   fpdt_tw_linear_*       the per-chunk QKV projection in front of the attention.
 *   fpdt_tw_ffn_*          the feed-forward block, chunked with twice the attention's chunk
 *                          count, forward and (recomputing) backward.
 *
 * The dense products run on this library's own bf16 MFMA kernels (csrc/tw_gemm.hip: operands
 * re-laid into MFMA fragments, 256 x 256 output tiles, fp32 accumulation); the row-wise softmax /
 * loss / gradient and the activations are HIP kernels of this library as well.  Built as a
 * separate shared library (libfpdt_tokenwise.so).
 *
 * Conventions as in fpdt.h: row-major contiguous tensors, device pointers, caller-owned
 * buffers, `stream` is a hipStream_t passed as void*, calls only enqueue, every function returns
 * an fpdt status code (0 = OK, 1 = invalid argument, 2 = unsupported, 3 = workspace, 4 = HIP
 * failure; text from fpdt_tw_last_error).  Besides the caller's workspace the library keeps one
 * device scratch pool per GPU for the re-laid operands of the running call (weights once per
 * call, activations per product); it grows on demand with hipMalloc -- so the first call of a
 * given size must not run under stream capture -- and is kept until the process ends.  Calls
 * that overlap in time on one GPU (different streams or threads) would share that pool: keep
 * the library's calls on one stream.
 */
#ifndef FPDT_TOKENWISE_H
#define FPDT_TOKENWISE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of device workspace fpdt_tw_loss_fwd_bwd needs: one chunk of fp32 logits and one chunk
 * of bf16 logit gradients, chunk = ceil(rows / n_chunks) rows.  0 if the arguments are invalid. */
size_t fpdt_tw_loss_workspace_bytes(int64_t rows, int hidden, int vocab, int n_chunks);

/*
 * Chunked cross-entropy loss with its output projection (Sec. 5.4).  For every row r:
 *     logits_r = H_r W^T                      (bf16 x bf16 -> fp32)
 *     lse_r    = log sum_v exp(logits_r[v])   (fp32, max-subtracted)
 *     loss_r   = lse_r - logits_r[target_r]
 * and, when dH / dW are given, the gradient of sum_r grad_scale * loss_r:
 *     G_r  = grad_scale * (softmax(logits_r) - onehot(target_r))    (rounded to bf16)
 *     dH_r = G_r W                            (written, bf16)
 *     dW  += G^T H                            (ACCUMULATED into the caller's fp32 buffer)
 *   H [rows, hidden] bf16, W [vocab, hidden] bf16, target [rows] int32 in [0, vocab)   in
 *   loss, lse [rows] fp32                                                             out
 *   dH [rows, hidden] bf16 or NULL, dW [vocab, hidden] fp32 or NULL                   out / in-out
 *   workspace: device memory, 256-byte aligned, >= fpdt_tw_loss_workspace_bytes(...)
 * A target outside [0, vocab) is not detected (its row's loss is lse_r and its gradient the
 * plain softmax).
 */
int fpdt_tw_loss_fwd_bwd(const void *H, const void *W, const int32_t *target, float grad_scale,
                         float *loss, float *lse, void *dH, float *dW, int64_t rows, int hidden,
                         int vocab, int n_chunks, void *workspace, size_t workspace_bytes,
                         void *stream);

/*
 * Chunked linear projection (Sec. 4.1: every sequence chunk T_i is projected to q_i, k_i, v_i on
 * its own, so that chunk i's attention can start while chunk i+1 is still being projected).
 *     Y = X W^T          X [rows, n_in] bf16, W [n_out, n_in] bf16  ->  Y [rows, n_out] bf16
 * computed ceil(rows / n_chunks) rows at a time; needs no workspace.  Backward:
 *     dX = dY W  (written, bf16; NULL to skip),   dW += dY^T X  (accumulated, fp32; NULL to skip)
 */
int fpdt_tw_linear_fwd(const void *X, const void *W, void *Y, int64_t rows, int n_in, int n_out,
                       int n_chunks, void *stream);
int fpdt_tw_linear_bwd(const void *X, const void *W, const void *dY, void *dX, float *dW,
                       int64_t rows, int n_in, int n_out, int n_chunks, void *stream);

/*
 * Chunked feed-forward block (Sec. 5.4: token-wise, its [rows, n_ffn] intermediates are what has
 * to be bounded; twice the attention's chunk count is enough, and nothing is offloaded).
 *   FPDT_TW_GELU    Y = gelu(X W1^T) W2^T                      (GPT; exact erf form)
 *   FPDT_TW_SWIGLU  Y = (silu(X W1^T) * (X W3^T)) W2^T         (Llama)
 *   X, Y, dX, dY [rows, n_model] bf16; W1, W3 [n_ffn, n_model] bf16; W2 [n_model, n_ffn] bf16
 *   (W3, dW3: SWIGLU only, NULL otherwise).  Intermediates are rounded to bf16 between GEMMs.
 * The backward recomputes the pre-activations of a chunk from X (the forward saves nothing),
 * writes dX and ACCUMULATES into the caller's fp32 dW1, dW3, dW2 (each may be NULL to skip).
 *   workspace: device memory, 256-byte aligned, >= fpdt_tw_ffn_workspace_bytes(..., is_bwd)
 */
enum { FPDT_TW_GELU = 0, FPDT_TW_SWIGLU = 1 };
size_t fpdt_tw_ffn_workspace_bytes(int64_t rows, int n_model, int n_ffn, int act, int n_chunks,
                                   int is_bwd);
int fpdt_tw_ffn_fwd(const void *X, const void *W1, const void *W3, const void *W2, void *Y,
                    int64_t rows, int n_model, int n_ffn, int act, int n_chunks, void *workspace,
                    size_t workspace_bytes, void *stream);
int fpdt_tw_ffn_bwd(const void *X, const void *W1, const void *W3, const void *W2, const void *dY,
                    void *dX, float *dW1, float *dW3, float *dW2, int64_t rows, int n_model,
                    int n_ffn, int act, int n_chunks, void *workspace, size_t workspace_bytes,
                    void *stream);

/* Text describing the calling thread's most recent error ("" if none). Never NULL. */
const char *fpdt_tw_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FPDT_TOKENWISE_H */
