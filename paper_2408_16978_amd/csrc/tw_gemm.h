// Dense bf16 products of the token-wise library (tw_gemm.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fpdt_tw {

// Start of a library call: forget the packed weights of the previous call and reuse its scratch.
void begin_call();

// C[M,N] (+)= sum_k Aop[m,k] * Bop[n,k], bf16 operands, fp32 accumulation.
//   a_transposed = 0: A is stored [M,K] (leading dimension lda); 1: A is stored [K,M]
//   b_transposed = 0: B is stored [N,K] (ldb);                   1: B is stored [K,N]
//   C row-major [M,N], leading dimension ldc, bf16 or fp32 (c_f32); accumulate: C += instead of C =
//   cache_b: B is a weight that further products of this library call will use again
// Only enqueues on `st`.  Returns 0, 1 (HIP failure) or 2 (sizes beyond the launch limits).
int gemm(int a_transposed, int b_transposed, int M, int N, int K, const void* A, int64_t lda, const void* B,
         int64_t ldb, void* C, int64_t ldc, bool c_f32, bool accumulate, bool cache_b, hipStream_t st);

}  // namespace fpdt_tw
