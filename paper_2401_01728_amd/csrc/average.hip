// Cluster average: the arithmetic of Parallel Multi-Ring All-Reduce (paper section 3.2,
// built on the ring all-reduce of section 2.3) for C replicas resident in one HBM.
//
// The network rounds disappear on one GPU; what remains of the algorithm is the
// partition (ring -> segment -> C chunks) and the order of the additions: chunk j is
// accumulated starting at replica j and walking the ring, then divided by C once.
// Each input element is read exactly once and each output written once, so the kernel
// is bound by HBM: (C+1)*4 bytes per element (+4 with a folded-in gradient; 2C*4 with
// write-back).
//
// Layout: one workgroup owns TILE consecutive elements.  Chunks are millions of
// elements long, so almost every tile lies inside one chunk: its rotation j is
// wave-uniform, the C replica base pointers are fetched with scalar loads in rotated
// order and each lane streams C independent 16-byte loads before the first add.
// Tiles that straddle a chunk boundary, the ragged tail and unaligned buffers take an
// element-wise path that computes the owning chunk per element.
#include "common.h"

#define RV_MAX_C 64
#define RV_MAX_R 4096

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

struct RepTable {
  float* p[RV_MAX_C];
};

constexpr int kThreads = 256;
constexpr int kVecPerThread = 2;                       // float4 per lane
constexpr int kTile = kThreads * kVecPerThread * 4;    // elements per workgroup

// Owning chunk of element i: ring r = ceil((i+1) R / n) - 1, then the same rule inside
// the ring's segment.
__device__ __forceinline__ int chunk_of(uint64_t i, uint64_t n, int R, int C) {
  uint64_t r = ((i + 1) * (uint64_t)R - 1) / n;
  uint64_t lo = (r * n) / (uint64_t)R;
  uint64_t hi = ((r + 1) * n) / (uint64_t)R;
  uint64_t s = hi - lo;
  return (int)(((i - lo + 1) * (uint64_t)C - 1) / s);
}

__device__ __forceinline__ float elem_mean(const RepTable& tab, int C, int j, uint64_t i,
                                           const float* grad, int gr, float eta) {
  float acc = 0.f;
  for (int s = 0; s < C; ++s) {
    int c = j + s; if (c >= C) c -= C;
    float v = tab.p[c][i];
    if (grad != nullptr && c == gr) v = __fsub_rn(v, __fmul_rn(grad[i], eta));
    acc = (s == 0) ? v : __fadd_rn(acc, v);
  }
  return __fdiv_rn(acc, (float)C);
}

template <int C, bool HAS_GRAD>
__device__ __forceinline__ void tile_fast(const RepTable& tab, int j, uint64_t base, float* out,
                                          int write_back, const float* grad, int gr, float eta) {
  const float invC_num = (float)C;
  f4 v[kVecPerThread][C];
#pragma unroll
  for (int u = 0; u < kVecPerThread; ++u) {
    uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
#pragma unroll
    for (int s = 0; s < C; ++s) {
      int c = j + s; if (c >= C) c -= C;
      c = __builtin_amdgcn_readfirstlane(c);
      const f4* p = reinterpret_cast<const f4*>(tab.p[c] + e);
      v[u][s] = __builtin_nontemporal_load(p);
      if (HAS_GRAD && c == gr) {
        f4 g = __builtin_nontemporal_load(reinterpret_cast<const f4*>(grad + e));
        v[u][s].x = __fsub_rn(v[u][s].x, __fmul_rn(g.x, eta));
        v[u][s].y = __fsub_rn(v[u][s].y, __fmul_rn(g.y, eta));
        v[u][s].z = __fsub_rn(v[u][s].z, __fmul_rn(g.z, eta));
        v[u][s].w = __fsub_rn(v[u][s].w, __fmul_rn(g.w, eta));
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kVecPerThread; ++u) {
    uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
    f4 a = v[u][0];
#pragma unroll
    for (int s = 1; s < C; ++s) {
      a.x = __fadd_rn(a.x, v[u][s].x);
      a.y = __fadd_rn(a.y, v[u][s].y);
      a.z = __fadd_rn(a.z, v[u][s].z);
      a.w = __fadd_rn(a.w, v[u][s].w);
    }
    a.x = __fdiv_rn(a.x, invC_num);
    a.y = __fdiv_rn(a.y, invC_num);
    a.z = __fdiv_rn(a.z, invC_num);
    a.w = __fdiv_rn(a.w, invC_num);
    if (out != nullptr) __builtin_nontemporal_store(a, reinterpret_cast<f4*>(out + e));
    if (write_back) {
#pragma unroll
      for (int c = 0; c < C; ++c)
        __builtin_nontemporal_store(a, reinterpret_cast<f4*>(tab.p[c] + e));
    }
  }
}

// C == 0 instantiates the generic (runtime-C) kernel, which only has the element path.
template <int CT, bool HAS_GRAD>
__global__ __launch_bounds__(kThreads) void average_kernel(RepTable tab, int Crt, uint64_t n, int R,
                                                           float* out, int write_back,
                                                           const float* grad, int gr, float eta,
                                                           int aligned) {
  const int C = CT > 0 ? CT : Crt;
  const uint64_t base = (uint64_t)blockIdx.x * kTile;
  __shared__ int sh_first, sh_last;
  if (threadIdx.x == 0) {
    uint64_t last = base + kTile - 1;
    sh_first = chunk_of(base, n, R, C);
    sh_last = last < n ? chunk_of(last, n, R, C) : -1;
    // a tile may also cross a ring boundary while staying in "chunk j" of two rings
    if (last < n) {
      uint64_t r0 = ((base + 1) * (uint64_t)R - 1) / n, r1 = ((last + 1) * (uint64_t)R - 1) / n;
      if (r0 != r1) sh_last = -1;
    }
  }
  __syncthreads();
  const int jf = sh_first, jl = sh_last;
  if constexpr (CT > 0) {
    if (aligned && jf == jl) {
      tile_fast<CT, HAS_GRAD>(tab, jf, base, out, write_back, grad, gr, eta);
      return;
    }
  }
  for (int k = threadIdx.x; k < kTile; k += kThreads) {
    uint64_t i = base + k;
    if (i >= n) break;
    int j = chunk_of(i, n, R, C);
    float m = elem_mean(tab, C, j, i, HAS_GRAD ? grad : nullptr, gr, eta);
    if (out != nullptr) out[i] = m;
    if (write_back)
      for (int c = 0; c < C; ++c) tab.p[c][i] = m;
  }
}

template <int CT>
void launch(const RepTable& tab, int C, uint64_t n, int R, float* out, int wb, const float* grad,
            int gr, float eta, int aligned, hipStream_t st) {
  unsigned blocks = (unsigned)((n + kTile - 1) / kTile);
  if (grad)
    hipLaunchKernelGGL((average_kernel<CT, true>), dim3(blocks), dim3(kThreads), 0, st, tab, C, n, R,
                       out, wb, grad, gr, eta, aligned);
  else
    hipLaunchKernelGGL((average_kernel<CT, false>), dim3(blocks), dim3(kThreads), 0, st, tab, C, n, R,
                       out, wb, grad, gr, eta, aligned);
}

}  // namespace

extern "C" rv_status rv_cluster_average(float* const* replicas, int C, size_t n, int R,
                                        float* mean_out, int write_back, const float* grad,
                                        int grad_replica, float eta, void* stream) {
  if (replicas == nullptr || C < 1 || C > RV_MAX_C || R < 1 || R > RV_MAX_R || n == 0)
    return RV_E_INVAL;
  if (mean_out == nullptr && !write_back) return RV_E_INVAL;
  if (grad != nullptr && (grad_replica < 0 || grad_replica >= C)) return RV_E_INVAL;
  if (n > ((uint64_t)1 << 40)) return RV_E_INVAL;   // keeps (i+1)*R inside 64 bits
  RepTable tab;
  int aligned = 1;
  for (int c = 0; c < C; ++c) {
    if (replicas[c] == nullptr) return RV_E_INVAL;
    for (int k = 0; k < c; ++k)
      if (replicas[k] == replicas[c]) return RV_E_INVAL;
    if (replicas[c] == mean_out) return RV_E_INVAL;
    tab.p[c] = replicas[c];
    if (((uintptr_t)replicas[c]) & 15) aligned = 0;
  }
  for (int c = C; c < RV_MAX_C; ++c) tab.p[c] = nullptr;
  if (mean_out && (((uintptr_t)mean_out) & 15)) aligned = 0;
  if (grad && (((uintptr_t)grad) & 15)) aligned = 0;
  hipStream_t st = (hipStream_t)stream;
  int wb = write_back ? 1 : 0;
  switch (C) {
    case 1: launch<1>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    case 2: launch<2>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    case 3: launch<3>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    case 4: launch<4>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    case 8: launch<8>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    case 16: launch<16>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
    default: launch<0>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, st); break;
  }
  return rv_launch_status();
}
