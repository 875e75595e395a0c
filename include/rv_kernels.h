/*
 * rv_kernels.h - per-kernel entry points of librv.so, for parity tests and profiling of
 * the individual steps of the decoder stage.  The product API is rv.h; these calls expose
 * the same kernels the stage launches, one at a time.  All pointers are device memory,
 * 16-byte aligned; every call enqueues on `stream` and returns without synchronising;
 * RV_E_INVAL on shapes the kernels do not cover.
 */
#ifndef RV_KERNELS_H
#define RV_KERNELS_H

#include "rv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Epilogues of the bf16 matrix product. */
enum {
  RV_EPI_BF16 = 0,               /* out bf16 = acc                                          */
  RV_EPI_BF16_BIAS = 1,          /* out bf16 = acc + bias[n]                                */
  RV_EPI_F32_BIAS_RESID = 2,     /* out f32  = acc + bias[n] + resid[m,n]                   */
  RV_EPI_BF16_BIAS_GELU = 3,     /* out bf16 = z = acc + bias[n]; out2 bf16 = GELU(z)       */
  RV_EPI_BF16_DGELU = 4,         /* out bf16 = acc * GELU'(zin[m,n])                        */
  RV_EPI_F32 = 5,                /* out f32  = acc                                          */
  RV_EPI_F32_BIAS_RESID_BF16 = 6 /* as 2, plus out2 bf16 = the same value rounded           */
};

/*
 * C[M,N] = sum_k A(m,k) B(k,n), bf16 operands, fp32 accumulation (the forward, input-
 * gradient and weight-gradient products of a Linear layer inside a peer's forward_pass
 * and its gradient, paper Alg. 1 / Eq. 2).
 *   a_kmajor = 0: A[m*lda + k];  1: A[k*lda + m].   b_kmajor = 0: B[n*ldb + k];  1: B[k*ldb + n].
 *   Supported (a_kmajor, b_kmajor, epilogue): (0,1,{1,2,3,6}), (0,0,{0,4}), (1,1,{5}).
 *   K % 64 == 0; M, N, lda, ldb % 8 == 0; ldo, ldr % 4 == 0.  tile: 0 = automatic, 128, 256.
 */
rv_status rv_k_gemm_bf16(const void* A, int64_t lda, int a_kmajor, const void* B, int64_t ldb,
                         int b_kmajor, int M, int N, int K, int epilogue, void* out, int64_t ldo,
                         void* out2, const void* bias, const float* resid, int64_t ldr,
                         const void* zin, int tile, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RV_KERNELS_H */
