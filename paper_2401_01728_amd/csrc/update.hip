// Delayed block SGD update (paper Eq. 2; Eq. 4 restricts it to the peer's own block):
// w <- w - eta * g on the flat fp32 master vector, one fused multiply-add per element,
// optionally emitting the new weights as the next weight version (bf16 for the
// decoder's matrix products, fp32 for the MLP stage).
//
// HBM-bound streaming kernel: reads w and g (4+4 B), writes w (4 B) and the version
// copy (2 or 4 B) per parameter.  16-byte accesses, one vector per lane and as many workgroups
// as tiles (measured best: 5.8 TB/s with the bf16 copy, 6.5 without).  A decoder stage taking the
// plain step does not come here: its update happens in the kernels that produce the gradient.
#include "common.h"
#include "internal.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kVec = 1;
constexpr int kTile = kThreads * kVec * 4;

// COPY: 0 none, 1 bf16, 2 fp32.  Without the bf16 version w and g stream through with non-temporal
// accesses (nothing is read twice; measured 76 % -> 81 % of HBM peak).  With it, only g does: every
// non-temporal access to w or to the version measured 3-5 % slower there (73 % -> 69-70 %), and so
// did 8 consecutive parameters per lane for a 16-byte bf16 store (the lanes of a wave must stay
// 16 bytes apart on w and g).
template <int COPY>
__global__ __launch_bounds__(kThreads) void update_kernel(float* __restrict__ w,
                                                          const float* __restrict__ g, uint64_t n,
                                                          float eta, void* __restrict__ copy,
                                                          int aligned) {
  const uint64_t base = (uint64_t)blockIdx.x * kTile;
  if (aligned && base + kTile <= n) {
    f4 wv[kVec], gv[kVec];
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
      uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
      if (COPY == 1) wv[u] = *reinterpret_cast<const f4*>(w + e);
      else wv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(w + e));
      gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
    }
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
      uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
      f4 r;
      r.x = __fmaf_rn(-eta, gv[u].x, wv[u].x);
      r.y = __fmaf_rn(-eta, gv[u].y, wv[u].y);
      r.z = __fmaf_rn(-eta, gv[u].z, wv[u].z);
      r.w = __fmaf_rn(-eta, gv[u].w, wv[u].w);
      if (COPY == 1) *reinterpret_cast<f4*>(w + e) = r;
      else __builtin_nontemporal_store(r, reinterpret_cast<f4*>(w + e));
      if (COPY == 1) {
        u2 pk;
        pk.x = rv_pack_bf16x2(r.x, r.y);
        pk.y = rv_pack_bf16x2(r.z, r.w);
        *reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(copy) + e) = pk;
      } else if (COPY == 2) {
        __builtin_nontemporal_store(r, reinterpret_cast<f4*>(reinterpret_cast<float*>(copy) + e));
      }
    }
    return;
  }
  for (int k = threadIdx.x; k < kTile; k += kThreads) {
    uint64_t i = base + k;
    if (i >= n) break;
    float r = __fmaf_rn(-eta, g[i], w[i]);
    w[i] = r;
    if (COPY == 1) reinterpret_cast<uint16_t*>(copy)[i] = rv_f32_to_bf16(r);
    if (COPY == 2) reinterpret_cast<float*>(copy)[i] = r;
  }
}

// The optimiser of the paper's single-cluster experiments (section 4.1: SGD with momentum
// 0.9 and weight decay 5e-4) as a variant of the same update, in the usual form
//   d = g + wd * w;   v <- mu * v + d;   w <- w - eta * v
// (three fused multiply-adds per element; wd = mu = 0 gives Eq. 2 bit for bit).
// 22 B/param with a bf16 copy: reads w, g, v, writes w, v, copy.
template <int COPY>
__global__ __launch_bounds__(kThreads) void update_momentum_kernel(float* __restrict__ w,
                                                                   const float* __restrict__ g,
                                                                   float* __restrict__ v, uint64_t n,
                                                                   float eta, float mu, float wd,
                                                                   void* __restrict__ copy, int aligned) {
  const uint64_t base = (uint64_t)blockIdx.x * kTile;
  auto step = [&](float wi, float gi, float& vi) {
    const float d = __fmaf_rn(wd, wi, gi);
    vi = __fmaf_rn(mu, vi, d);
    return __fmaf_rn(-eta, vi, wi);
  };
  if (aligned && base + kTile <= n) {
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
      const uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
      const f4 wv = *reinterpret_cast<const f4*>(w + e);
      const f4 gv = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
      f4 vv = *reinterpret_cast<const f4*>(v + e);
      f4 r;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float vi = vv[c];
        r[c] = step(wv[c], gv[c], vi);
        vv[c] = vi;
      }
      *reinterpret_cast<f4*>(w + e) = r;
      *reinterpret_cast<f4*>(v + e) = vv;
      if (COPY == 1) {
        u2 pk;
        pk.x = rv_pack_bf16x2(r.x, r.y);
        pk.y = rv_pack_bf16x2(r.z, r.w);
        *reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(copy) + e) = pk;
      } else if (COPY == 2) {
        *reinterpret_cast<f4*>(reinterpret_cast<float*>(copy) + e) = r;
      }
    }
    return;
  }
  for (int k = threadIdx.x; k < kTile; k += kThreads) {
    const uint64_t i = base + k;
    if (i >= n) break;
    float vi = v[i];
    const float r = step(w[i], g[i], vi);
    w[i] = r; v[i] = vi;
    if (COPY == 1) reinterpret_cast<uint16_t*>(copy)[i] = rv_f32_to_bf16(r);
    if (COPY == 2) reinterpret_cast<float*>(copy)[i] = r;
  }
}

// Gradient accumulation (section 4.2 of the paper: the gradients of several microbatches are
// summed before one update): acc <- g for the first microbatch of a group, acc <- acc + g
// after.  12 B/param (8 for the first).
template <bool FIRST>
__global__ __launch_bounds__(kThreads) void accumulate_kernel(float* __restrict__ acc, const float* __restrict__ g,
                                                              uint64_t n, int aligned) {
  const uint64_t base = (uint64_t)blockIdx.x * kTile;
  if (aligned && base + kTile <= n) {
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
      const uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
      f4 gv = *reinterpret_cast<const f4*>(g + e);
      if (!FIRST) gv += *reinterpret_cast<const f4*>(acc + e);
      *reinterpret_cast<f4*>(acc + e) = gv;
    }
    return;
  }
  for (int k = threadIdx.x; k < kTile; k += kThreads) {
    const uint64_t i = base + k;
    if (i >= n) break;
    acc[i] = FIRST ? g[i] : acc[i] + g[i];
  }
}

// plain conversion of the master vector into a version slot (set_params)
template <int COPY>
__global__ __launch_bounds__(kThreads) void publish_kernel(const float* __restrict__ w, uint64_t n,
                                                           void* __restrict__ copy) {
  uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n) return;
  if (COPY == 1) reinterpret_cast<uint16_t*>(copy)[i] = rv_f32_to_bf16(w[i]);
  if (COPY == 2) reinterpret_cast<float*>(copy)[i] = w[i];
}

}  // namespace

rv_status rv_launch_update(float* w, const float* g, size_t n, float eta, void* copy, int copy_kind,
                           hipStream_t st) {
  if (n == 0) return RV_OK;
  int aligned = ((((uintptr_t)w) | ((uintptr_t)g)) & 15) == 0;
  if (copy && (((uintptr_t)copy) & 15)) aligned = 0;
  unsigned blocks = (unsigned)((n + kTile - 1) / kTile);
  if (!copy || copy_kind == 0)
    hipLaunchKernelGGL(update_kernel<0>, dim3(blocks), dim3(kThreads), 0, st, w, g, n, eta, nullptr, aligned);
  else if (copy_kind == 1)
    hipLaunchKernelGGL(update_kernel<1>, dim3(blocks), dim3(kThreads), 0, st, w, g, n, eta, copy, aligned);
  else
    hipLaunchKernelGGL(update_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, w, g, n, eta, copy, aligned);
  return rv_launch_status();
}

rv_status rv_launch_update_momentum(float* w, const float* g, float* v, size_t n, float eta, float mu, float wd,
                                    void* copy, int copy_kind, hipStream_t st) {
  if (n == 0) return RV_OK;
  int aligned = ((((uintptr_t)w) | ((uintptr_t)g) | ((uintptr_t)v)) & 15) == 0;
  if (copy && (((uintptr_t)copy) & 15)) aligned = 0;
  unsigned blocks = (unsigned)((n + kTile - 1) / kTile);
  if (!copy || copy_kind == 0)
    hipLaunchKernelGGL(update_momentum_kernel<0>, dim3(blocks), dim3(kThreads), 0, st, w, g, v, n, eta, mu, wd, nullptr, aligned);
  else if (copy_kind == 1)
    hipLaunchKernelGGL(update_momentum_kernel<1>, dim3(blocks), dim3(kThreads), 0, st, w, g, v, n, eta, mu, wd, copy, aligned);
  else
    hipLaunchKernelGGL(update_momentum_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, w, g, v, n, eta, mu, wd, copy, aligned);
  return rv_launch_status();
}

rv_status rv_launch_accumulate(float* acc, const float* g, size_t n, bool first, hipStream_t st) {
  if (n == 0) return RV_OK;
  const int aligned = ((((uintptr_t)acc) | ((uintptr_t)g)) & 15) == 0;
  const unsigned blocks = (unsigned)((n + kTile - 1) / kTile);
  if (first) hipLaunchKernelGGL(accumulate_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, acc, g, n, aligned);
  else hipLaunchKernelGGL(accumulate_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, acc, g, n, aligned);
  return rv_launch_status();
}

rv_status rv_launch_publish(const float* w, size_t n, void* copy, int copy_kind, hipStream_t st) {
  if (n == 0) return RV_OK;
  unsigned blocks = (unsigned)((n + kThreads - 1) / kThreads);
  if (copy_kind == 1)
    hipLaunchKernelGGL(publish_kernel<1>, dim3(blocks), dim3(kThreads), 0, st, w, n, copy);
  else
    hipLaunchKernelGGL(publish_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, w, n, copy);
  return rv_launch_status();
}

extern "C" rv_status rv_block_update(float* w, const float* g, size_t n, float eta, void* bf16_out,
                                     void* stream) {
  if (w == nullptr || g == nullptr || n == 0) return RV_E_INVAL;
  if ((const float*)w == g) return RV_E_INVAL;
  return rv_launch_update(w, g, n, eta, bf16_out, bf16_out ? 1 : 0, (hipStream_t)stream);
}

extern "C" rv_status rv_block_update_momentum(float* w, const float* g, float* v, size_t n, float eta,
                                              float momentum, float weight_decay, void* bf16_out, void* stream) {
  if (w == nullptr || g == nullptr || v == nullptr || n == 0) return RV_E_INVAL;
  if ((const float*)w == g || (const float*)v == g || w == v) return RV_E_INVAL;
  if (!(momentum >= 0.f) || !(weight_decay >= 0.f)) return RV_E_INVAL;
  return rv_launch_update_momentum(w, g, v, n, eta, momentum, weight_decay, bf16_out, bf16_out ? 1 : 0,
                                   (hipStream_t)stream);
}
