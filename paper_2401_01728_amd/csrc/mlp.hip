// fp32 MLP stage (Linear -> ReLU -> ... -> Linear): the forward_pass of a peer in the
// paper's Alg. 1 and its exact gradient, for stages small enough that launch latency,
// not arithmetic, bounds them.  Plain LDS-tiled fp32 products with a fixed summation
// order (deterministic).
//
// Stash per microbatch: the input of every Linear (a_0 .. a_{n-1}).  Because a_{i+1} =
// ReLU(z_i), "a_{i+1} > 0" is the ReLU gate of layer i, so pre-activations are not kept.
#include "internal.h"

namespace {

struct MlpPlan {
  int n = 0;
  std::vector<size_t> offW, offB;   // into the flat parameter vector
  std::vector<size_t> offA;         // a_i inside a stash slot (floats)
  size_t maxw = 0;
};

constexpr int TS = 16;

// C[M,N] = sum_k A(m,k) * B(k,n) with element strides; epilogue:
//   bias != null : + bias[n];  relu : max(.,0);  gate != null : * (gate[m*N+n] > 0)
__global__ __launch_bounds__(TS * TS) void gemm_f32_kernel(const float* __restrict__ A, int64_t sAm,
                                                           int64_t sAk, const float* __restrict__ B,
                                                           int64_t sBk, int64_t sBn,
                                                           float* __restrict__ Cm, int M, int N,
                                                           int K, const float* __restrict__ bias,
                                                           int relu, const float* __restrict__ gate) {
  __shared__ float As[TS][TS + 1];
  __shared__ float Bs[TS][TS + 1];
  const int tx = threadIdx.x % TS, ty = threadIdx.x / TS;
  const int m = blockIdx.y * TS + ty, n = blockIdx.x * TS + tx;
  float acc = 0.f;
  for (int k0 = 0; k0 < K; k0 += TS) {
    int ka = k0 + tx, kb = k0 + ty;
    As[ty][tx] = (m < M && ka < K) ? A[m * sAm + ka * sAk] : 0.f;
    Bs[ty][tx] = (kb < K && n < N) ? B[kb * sBk + n * sBn] : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TS; ++k) acc = __fmaf_rn(As[ty][k], Bs[k][tx], acc);
    __syncthreads();
  }
  if (m < M && n < N) {
    if (bias) acc += bias[n];
    if (relu) acc = fmaxf(acc, 0.f);
    if (gate) acc = gate[(int64_t)m * N + n] > 0.f ? acc : 0.f;
    Cm[(int64_t)m * N + n] = acc;
  }
}

// out[n] = sum_m D[m,n]  (rows summed in order)
__global__ void colsum_f32_kernel(const float* __restrict__ D, int M, int N, float* __restrict__ out) {
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float acc = 0.f;
  for (int m = 0; m < M; ++m) acc += D[(int64_t)m * N + n];
  out[n] = acc;
}

void gemm(hipStream_t st, const float* A, int64_t sAm, int64_t sAk, const float* B, int64_t sBk,
          int64_t sBn, float* C, int M, int N, int K, const float* bias, int relu, const float* gate) {
  dim3 grid((N + TS - 1) / TS, (M + TS - 1) / TS);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(TS * TS), 0, st, A, sAm, sAk, B, sBk, sBn, C, M, N, K,
                     bias, relu, gate);
}

}  // namespace

rv_status rv_mlp_plan(rv_stage* s) {
  MlpPlan* p = new (std::nothrow) MlpPlan();
  if (!p) return RV_E_NOMEM;
  s->impl = p;
  p->n = s->n_layers;
  size_t off = 0, offa = 0;
  for (int i = 0; i <= p->n; ++i) {
    if (s->dims[i] < 1 || s->dims[i] > (1 << 20)) return RV_E_INVAL;
    p->maxw = std::max(p->maxw, (size_t)s->dims[i]);
  }
  for (int i = 0; i < p->n; ++i) {
    p->offW.push_back(off); off += (size_t)s->dims[i] * s->dims[i + 1];
    p->offB.push_back(off); off += (size_t)s->dims[i + 1];
    p->offA.push_back(offa); offa += (size_t)s->microbatch * s->dims[i];
  }
  s->P = off;
  s->slot_bytes = offa * 4;
  s->work_bytes = 2 * (size_t)s->microbatch * p->maxw * 4;
  return RV_OK;
}

void rv_mlp_free(rv_stage* s) {
  delete (MlpPlan*)s->impl;
  s->impl = nullptr;
}

rv_status rv_mlp_forward(rv_stage* s, rv_slot& slot, const void* in, void* out) {
  MlpPlan* p = (MlpPlan*)s->impl;
  const float* w = (const float*)s->ver[slot.ver];
  float* stash = (float*)slot.base;
  const int mb = s->microbatch;
  RV_HIP_TRY(hipMemcpyAsync(stash + p->offA[0], in, (size_t)mb * s->dims[0] * 4,
                            hipMemcpyDeviceToDevice, s->st));
  for (int i = 0; i < p->n; ++i) {
    const bool last = i == p->n - 1;
    float* dst = last ? (float*)out : stash + p->offA[i + 1];
    const int K = (int)s->dims[i], N = (int)s->dims[i + 1];
    gemm(s->st, stash + p->offA[i], K, 1, w + p->offW[i], N, 1, dst, mb, N, K, w + p->offB[i],
         last ? 0 : 1, nullptr);
  }
  return rv_launch_status();
}

rv_status rv_mlp_backward(rv_stage* s, rv_slot& slot, const void* grad_out, void* grad_in) {
  MlpPlan* p = (MlpPlan*)s->impl;
  const float* w = (const float*)s->ver[slot.ver];
  const float* stash = (const float*)slot.base;
  const int mb = s->microbatch;
  float* ping = (float*)s->work;
  float* pong = ping + (size_t)mb * p->maxw;
  const float* d = (const float*)grad_out;   // dL/dz_i, already gated
  for (int i = p->n - 1; i >= 0; --i) {
    const int K = (int)s->dims[i], N = (int)s->dims[i + 1];
    const float* a = stash + p->offA[i];
    // dW_i[K,N] = a_i^T d ; db_i = column sums of d
    gemm(s->st, a, 1, K, d, N, 1, s->grad + p->offW[i], K, N, mb, nullptr, 0, nullptr);
    hipLaunchKernelGGL(colsum_f32_kernel, dim3((N + 127) / 128), dim3(128), 0, s->st, d, mb, N,
                       s->grad + p->offB[i]);
    // d_{i-1}[mb,K] = (d W_i^T) gated by a_i > 0 (no gate in front of the first layer)
    if (i > 0 || grad_in) {
      float* dst = i == 0 ? (float*)grad_in : (d == ping ? pong : ping);
      gemm(s->st, d, N, 1, w + p->offW[i], 1, N, dst, mb, K, N, nullptr, 0, i > 0 ? a : nullptr);
      d = dst;
    }
  }
  return rv_launch_status();
}
