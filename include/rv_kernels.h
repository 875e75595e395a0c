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
 *   K % 64 == 0; M, N, lda, ldb % 8 == 0; ldo % 8 == 0 for bf16 outputs and % 4 for fp32 ones;
 *   ldr % 4 == 0.  tile: 0 = automatic; 2128 (128x128), 2192 (128x256), 2256 (256x256, four
 *   waves), 5256 (256x256, eight waves) force a tile.
 */
rv_status rv_k_gemm_bf16(const void* A, int64_t lda, int a_kmajor, const void* B, int64_t ldb,
                         int b_kmajor, int M, int N, int K, int epilogue, void* out, int64_t ldo,
                         void* out2, const void* bias, const float* resid, int64_t ldr,
                         const void* zin, int tile, void* stream);

/*
 * Up to 4 weight-gradient products dW_i[M_i,N_i] = X_i^T dY_i (both operands k-major: X_i is
 * [K, M_i] with pitch lda_i, dY_i is [K, N_i] with pitch ldb_i; fp32 outputs with pitch N_i)
 * over the same K tokens, in ONE launch: the four products of a decoder block together fill
 * the chip where each alone would not.  Arrays are HOST arrays of `count` entries; operand
 * pointers are device pointers.  Same divisibility rules as rv_k_gemm_bf16; results equal
 * rv_k_gemm_bf16(..., epilogue 5, tile 5256) bit for bit.
 */
rv_status rv_k_gemm_wgrad_grouped(int count, const void* const* X, const int64_t* lda, const void* const* dY,
                                  const int64_t* ldb, const int* M, const int* N, int K, float* const* dW,
                                  void* stream);

/*
 * LayerNorm over the last dimension (biased variance, eps inside the root), affine in
 * bf16: y bf16 [T,d] = (x - mean) * rstd * gamma + beta; mean, rstd fp32 [T] are kept for
 * the backward.  x is fp32 [T,d], or bf16 when x_is_bf16 (then xcopy receives it widened
 * to fp32).  d % 4 == 0, d <= 8192.
 */
rv_status rv_k_layernorm_fwd(const void* x, int x_is_bf16, float* xcopy, const void* gamma,
                             const void* beta, void* y, float* mean, float* rstd, int T, int d,
                             float eps, void* stream);

/*
 * Backward of the LayerNorm joined with the residual branch it hangs off:
 *   dx = dres + rstd * (dxh - mean(dxh) - xh * mean(dxh * xh)),  dxh = dy * gamma
 * dy bf16 [T,d]; x, dres, dx fp32 [T,d] (dx may alias dres); dx_bf16 optional bf16 copy.
 * Column sums over tokens: dgamma = sum dy*xh, dbeta = sum dy, dbias = sum dx (each fp32
 * [d], each optional).  part: scratch of ceil(T/8)*3*d floats.  d <= 4096.
 */
rv_status rv_k_layernorm_bwd(const void* dy, const float* x, const float* mean, const float* rstd,
                             const void* gamma, const float* dres, float* dx, void* dx_bf16,
                             float* part, float* dgamma, float* dbeta, float* dbias, int T, int d,
                             void* stream);

/*
 * Causal self-attention.  qkv bf16 [microbatch*seq, 3*d_model] (column thirds q|k|v, heads
 * contiguous inside a third); out bf16 [microbatch*seq, d_model];
 * lse2 fp32 [microbatch, n_heads, seq] = log2 of the softmax denominator in the scaled
 * base-2 domain (kept for the backward).  d_model/n_heads in {64,128}, seq % 64 == 0.
 */
rv_status rv_k_attention_fwd(const void* qkv, void* out, float* lse2, int microbatch, int seq,
                             int d_model, int n_heads, void* stream);
/* Gradient of the above: dout bf16 [T,d_model] -> dqkv bf16 [T,3*d_model];
 * dscratch: fp32 [microbatch*n_heads*seq]. */
rv_status rv_k_attention_bwd(const void* qkv, const void* out, const void* dout, const float* lse2,
                             float* dscratch, void* dqkv, int microbatch, int seq, int d_model,
                             int n_heads, void* stream);

/*
 * rv_k_attention_bwd for callers that cannot allocate or own a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the
 * per-row scratch (one float per (microbatch, head, position)) in a fixed 1 MiB device array
 * inside the library instead of `dscratch`.  The call allocates and frees nothing.
 * RV_E_INVAL when microbatch * n_heads * seq > 262144, and on the shapes rv_k_attention_bwd
 * rejects.  All calls on one GPU share that array: calls that overlap on one GPU (different
 * streams, or threads) race; calls on one stream are ordered and need no clearing in between.
 */
rv_status rv_k_attention_bwd_static(const void* qkv, const void* out, const void* dout, const float* lse2,
                                    void* dqkv, int microbatch, int seq, int d_model, int n_heads,
                                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RV_KERNELS_H */
