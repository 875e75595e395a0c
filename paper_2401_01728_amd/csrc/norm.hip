// LayerNorm forward / backward and the column reductions behind bias and LN-affine
// gradients of the decoder block (pieces of a peer's forward_pass and of its exact
// gradient, paper Alg. 1 / Eq. 2).  All HBM-bound: one wave owns a token row, a lane owns
// 16-byte column groups lane*4 + 256*i, statistics are reduced with wave shuffles, the
// residual stream and its gradient stay fp32, matrix-product operands leave as bf16.
//
// Column sums over tokens (bias and LayerNorm-affine gradients) are produced in two
// deterministic steps: the kernel that has the summands in hand - LayerNorm backward here, the
// attention backward and the GELU' epilogue of the matrix product elsewhere - writes one partial
// row per workgroup, and reduce_rows_kernel adds the partial rows in order (and applies the
// delayed update to those small parameter vectors on the spot).
#include "internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// The butterfly of wave_sum without lane-address registers: the two 32-lane halves are exchanged
// with v_permlane32_swap, the rest with ds_swizzle's immediate patterns.  Same pairs, same sums.
__device__ __forceinline__ float wave_sum_imm(float v) {
  const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(h[0]) + __uint_as_float(h[1]);
  v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), (16 << 10) | 0x1F));
  v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), (8 << 10) | 0x1F));
  v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), (4 << 10) | 0x1F));
  v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), (2 << 10) | 0x1F));
  v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), (1 << 10) | 0x1F));
  return v;
}

__device__ __forceinline__ f32x4 bf16x4_to_f32(u32x2 b) {
  f32x4 r;
  r.x = __uint_as_float(b.x << 16); r.y = __uint_as_float(b.x & 0xFFFF0000u);
  r.z = __uint_as_float(b.y << 16); r.w = __uint_as_float(b.y & 0xFFFF0000u);
  return r;
}
__device__ __forceinline__ u32x2 f32_to_bf16x4(f32x4 a) {
  u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
  return o;
}

// y = LN(x) * gamma + beta.  IN_BF16: x arrives as bf16 (stage input) and is also written
// out as the fp32 residual stream xcopy.
// Four waves of at most 80 registers (NV <= 8) and no LDS: such a workgroup still finds room on a
// CU whose registers are mostly held by two 200-register waves per SIMD of a matrix-product
// kernel of another stream, so the HBM-bound LayerNorm can run under the MFMA-bound products.
template <int NV, bool IN_BF16>
__global__ __launch_bounds__(kThreads, NV <= 8 ? 6 : 1) void ln_fwd_kernel(const void* __restrict__ xin,
                                                          float* __restrict__ xcopy,
                                                          const uint16_t* __restrict__ gamma,
                                                          const uint16_t* __restrict__ beta,
                                                          uint16_t* __restrict__ y,
                                                          float* __restrict__ mean,
                                                          float* __restrict__ rstd, int T, int d,
                                                          float eps) {
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int row = blockIdx.x * kWaves + wave;
  if (row >= T) return;
  f32x4 v[NV];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    // every lane loads (columns past the row's end re-read its last four and are zeroed): no
    // branch around a load, so all NV of them are in flight together
    const int c = l * 4 + 256 * i, cc = c < d ? c : d - 4;
    if (IN_BF16) v[i] = bf16x4_to_f32(*reinterpret_cast<const u32x2*>((const uint16_t*)xin + (int64_t)row * d + cc));
    else v[i] = *reinterpret_cast<const f32x4*>((const float*)xin + (int64_t)row * d + cc);
    if (c >= d) v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = l * 4 + 256 * i;
    if (IN_BF16 && c < d) *reinterpret_cast<f32x4*>(xcopy + (int64_t)row * d + c) = v[i];
    s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
  const float mu = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = l * 4 + 256 * i;
    if (c < d) {
      f32x4 t = v[i] - mu;
      q += (t.x * t.x + t.y * t.y) + (t.z * t.z + t.w * t.w);
    }
  }
  const float r = rsqrtf(wave_sum(q) / (float)d + eps);
  if (l == 0) { mean[row] = mu; rstd[row] = r; }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = l * 4 + 256 * i, cc = c < d ? c : d - 4;
    const f32x4 g = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(gamma + cc));
    const f32x4 b = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(beta + cc));
    const f32x4 o = (v[i] - mu) * r * g + b;
    if (c < d) *reinterpret_cast<u32x2*>(y + (int64_t)row * d + c) = f32_to_bf16x4(o);
  }
}

// The fp32-input forward with RPW rows per wave and two alternating sets of row registers: the
// next row is requested before the current one is reduced and stored, so a wave keeps two rows
// on the way instead of one.  Used up to d = 1792 (seven column groups: two sets fit the 96
// registers that are free beside a matrix-product kernel, but for nine spilled dwords; with eight
// groups the spills cost the 2048-wide stage step 1.6 %).  RPW is chosen so that a launch has about
// two workgroups per CU: 4 from 8192 rows on, else 2 - stage steps -0.5 % (d = 1600, 8192 rows)
// and -0.25 % (d = 1024, 4096 rows); the other choice measured +0.2 % / +0.3 %.
template <int NV, int RPW>
__global__ __launch_bounds__(kThreads, 5) void ln_fwd_pipe_kernel(const float* __restrict__ xin,
                                                                  const uint16_t* __restrict__ gamma,
                                                                  const uint16_t* __restrict__ beta,
                                                                  uint16_t* __restrict__ y,
                                                                  float* __restrict__ mean,
                                                                  float* __restrict__ rstd, int T, int d,
                                                                  float eps) {
  static_assert(RPW % 2 == 0, "rows alternate between two register sets");
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int row0 = (blockIdx.x * kWaves + wave) * RPW;
  if (row0 >= T) return;
  // byte offset of the lane's i-th fp32 column group in a row (clamped past the end); recomputed
  // where it is used: NV registers less
  auto cbo = [&](int i) -> unsigned {
    const int c = l * 4 + 256 * i;
    return (unsigned)(c < d ? c : d - 4) * 4u;
  };
  auto request = [&](f32x4 (&v)[NV], int row) {
    const char* xr = reinterpret_cast<const char*>(xin + (int64_t)(row < T ? row : T - 1) * d);
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = *reinterpret_cast<const f32x4*>(xr + cbo(i));
  };
  auto finish = [&](f32x4 (&v)[NV], int row) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      if (l * 4 + 256 * i >= d) v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    const float mu = wave_sum_imm(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      if (l * 4 + 256 * i < d) {
        f32x4 t = v[i] - mu;
        q += (t.x * t.x + t.y * t.y) + (t.z * t.z + t.w * t.w);
      }
    }
    const float r = rsqrtf(wave_sum_imm(q) / (float)d + eps);
    if (row >= T) return;
    if (l == 0) { mean[row] = mu; rstd[row] = r; }
    char* yr = reinterpret_cast<char*>(y + (int64_t)row * d);
    // gamma and beta are fetched again for every row (they stay in cache) rather than held in
    // 4 * NV registers across rows
    const char* gp = reinterpret_cast<const char*>(gamma);
    const char* bp = reinterpret_cast<const char*>(beta);
    asm volatile("" : "+s"(gp), "+s"(bp));
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const f32x4 g = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(gp + (cbo(i) >> 1)));
      const f32x4 b = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(bp + (cbo(i) >> 1)));
      const f32x4 o = (v[i] - mu) * r * g + b;
      if (l * 4 + 256 * i < d) *reinterpret_cast<u32x2*>(yr + (cbo(i) >> 1)) = f32_to_bf16x4(o);
      if (NV > 4 && i % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // gamma/beta of four column groups at a time
    }
  };
  f32x4 va[NV], vb[NV];
  request(va, row0);
#pragma unroll 1
  for (int k = 0; k < RPW - 2; k += 2) {
    request(vb, row0 + k + 1);
    finish(va, row0 + k);
    request(va, row0 + k + 2);
    finish(vb, row0 + k + 1);
  }
  request(vb, row0 + RPW - 1);
  finish(va, row0 + RPW - 2);
  finish(vb, row0 + RPW - 1);
}

// Backward of y = LN(x)*gamma + beta joined with the residual branch:
//   dx = dres + rstd * (dxh - mean(dxh) - xh * mean(dxh * xh)),  dxh = dy * gamma
// Writes dx (fp32, may alias dres) and optionally its bf16 rounding; accumulates three
// column sums over the workgroup's rows into part[blk][0..2][d]:
//   0: sum dy * xh (d gamma)   1: sum dy (d beta)   2: sum dx (bias gradient of the Linear
//   whose output fed this residual stream).
constexpr int kRowsPerBlock = 16;
constexpr int kBwdWaves = 4;

// Four waves per workgroup, all on the same rows: wave cs owns columns [cs * NV * 256, +NV * 256)
// of every row, a lane NV 16-byte column groups of them, and RF rows are in flight at once - all
// their operands are requested before the first is used, so a workgroup keeps RF * 10 * d bytes
// on the way instead of one row's.  What bounds the choice is 80 registers per lane: one such
// wave per SIMD (and a few hundred bytes of LDS) still fits beside the two ~210-register waves
// of a matrix-product kernel of another stream, so the HBM-bound backward runs under the
// MFMA-bound products instead of waiting for a free CU.  This kernel serves d > 1024: NV = 2,
// RF = 1 up to 2048; NV = 4 beyond (no such stage is benchmarked); d <= 1024 takes
// ln_bwd_pipe_kernel below, which keeps twice the rows in flight.  Row statistics are combined
// through LDS in a fixed order, one barrier per RF rows, two alternating slots.  The column sums
// stay in registers for the workgroup's 16 rows and leave as one partial row per workgroup.
template <int NV, int RF>
__global__ __launch_bounds__(64 * kBwdWaves, NV <= 2 ? 6 : 1) void ln_bwd_kernel(const uint16_t* __restrict__ dy,
                                                                const float* __restrict__ x,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ rstd,
                                                                const uint16_t* __restrict__ gamma,
                                                                const float* dres, float* dx,
                                                                uint16_t* __restrict__ dx_bf16,
                                                                float* __restrict__ part, int T, int d) {
  constexpr int CS = kBwdWaves;
  __shared__ float stat[2][RF][CS][2];
  const int cs = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int cbase = cs * (NV * 256) + l * 4;
  f32x4 ag[NV], ab[NV], ax[NV], gam[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    ag[i] = 0.f; ab[i] = 0.f; ax[i] = 0.f; gam[i] = 0.f;
    const int c = cbase + 256 * i;
    gam[i] = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(gamma + (c < d ? c : d - 4)));
    if (c >= d) gam[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll 1
  for (int k = 0; k < kRowsPerBlock / RF; ++k) {
    const int row0 = blockIdx.x * kRowsPerBlock + k * RF;
    // every operand of the RF rows is requested here: one memory round trip per RF rows
    f32x4 xh[RF][NV], rs[RF][NV];
    u32x2 dyr[RF][NV];
    float mu[RF], r[RF];
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      const int row = row0 + q;
      const bool valid = row < T;
      mu[q] = valid ? mean[row] : 0.f; r[q] = valid ? rstd[row] : 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = cbase + 256 * i;
        xh[q][i] = 0.f; rs[q][i] = 0.f; dyr[q][i] = u32x2{0u, 0u};
        if (valid && c < d) {
          // read once, written once: the non-temporal hint keeps these rows from pushing the
          // operand panels of the matrix products on the other streams out of L2
          xh[q][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + (int64_t)row * d + c));
          rs[q][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(dres + (int64_t)row * d + c));
          dyr[q][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(dy + (int64_t)row * d + c));
        }
      }
    }
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = cbase + 256 * i;
        if (c < d) {
          xh[q][i] = (xh[q][i] - mu[q]) * r[q];
          const f32x4 dxh = bf16x4_to_f32(dyr[q][i]) * gam[i];
          const f32x4 t = dxh * xh[q][i];
          s1 += (dxh.x + dxh.y) + (dxh.z + dxh.w);
          s2 += (t.x + t.y) + (t.z + t.w);
        }
      }
      s1 = wave_sum(s1); s2 = wave_sum(s2);
      if (l == 0) { stat[k & 1][q][cs][0] = s1; stat[k & 1][q][cs][1] = s2; }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      const int row = row0 + q;
      float s1 = stat[k & 1][q][0][0], s2 = stat[k & 1][q][0][1];
#pragma unroll
      for (int w = 1; w < CS; ++w) { s1 += stat[k & 1][q][w][0]; s2 += stat[k & 1][q][w][1]; }
      const float c1 = s1 / (float)d, c2 = s2 / (float)d;
      if (row < T) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int c = cbase + 256 * i;
          if (c < d) {
            const f32x4 dyv = bf16x4_to_f32(dyr[q][i]);
            const f32x4 dxh = dyv * gam[i];
            const f32x4 o = (dxh - c1 - xh[q][i] * c2) * r[q] + rs[q][i];
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(dx + (int64_t)row * d + c));
            if (dx_bf16) __builtin_nontemporal_store(f32_to_bf16x4(o), reinterpret_cast<u32x2*>(dx_bf16 + (int64_t)row * d + c));
            ag[i] += dyv * xh[q][i];
            ab[i] += dyv;
            ax[i] += o;
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = cbase + 256 * i;
    if (c < d) {
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 0) * d + c) = ag[i];
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 1) * d + c) = ab[i];
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 2) * d + c) = ax[i];
    }
  }
}

// The same arithmetic, in the same order, with the next RF rows' operands already requested
// while the current RF rows are reduced, combined and stored: two sets of row registers
// alternate, so 2 * RF rows are on the way per workgroup.  Beside a matrix-product kernel only
// one such workgroup fits on a CU, and what it has in flight is what bounds it.  For d <= 1024
// (NV = 1, RF = 2) both sets fit in 81 registers and the stage step of the 1024-wide stage
// measured 0.5 % shorter.  For 1024 < d <= 2048 two sets and the 24 column-sum registers do not
// fit in the 96 registers that are free beside two ~200-register waves; with the column sums
// moved to LDS they did, and the 1600-wide stage steps measured within +-0.2 % of
// ln_bwd_kernel<2, 1>, which therefore stays.
template <int NV, int RF>
struct LnRows {
  f32x4 xh[RF][NV], rs[RF][NV];
  u32x2 dy[RF][NV];
  float mu[RF], r[RF];
};
template <int NV, int RF, int ROWS>
__global__ __launch_bounds__(64 * kBwdWaves, 5) void ln_bwd_pipe_kernel(const uint16_t* __restrict__ dy,
                                                                const float* __restrict__ x,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ rstd,
                                                                const uint16_t* __restrict__ gamma,
                                                                const float* dres, float* dx,
                                                                uint16_t* __restrict__ dx_bf16,
                                                                float* __restrict__ part, int T, int d) {
  constexpr int CS = kBwdWaves;
  constexpr int G = ROWS / RF;
  static_assert(ROWS % RF == 0 && G % 2 == 0, "row groups alternate between two register sets");
  __shared__ float stat[2][RF][CS][2];
  const int cs = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int cbase = cs * (NV * 256) + l * 4;
  f32x4 ag[NV], ab[NV], ax[NV], gam[NV];
  unsigned cb[NV];   // byte offset of the lane's fp32 column group in a row
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    ag[i] = 0.f; ab[i] = 0.f; ax[i] = 0.f;
    const int c = cbase + 256 * i;
    cb[i] = (unsigned)(c < d ? c : d - 4) * 4u;
    gam[i] = bf16x4_to_f32(*reinterpret_cast<const u32x2*>(gamma + (cb[i] >> 2)));
    if (c >= d) gam[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // every lane loads: rows past the end re-read the last row, columns past the end the row's last
  // four; neither is used
  auto request = [&](LnRows<NV, RF>& w, int row0) {
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      const int row = row0 + q < T ? row0 + q : T - 1;
      w.mu[q] = mean[row]; w.r[q] = rstd[row];
      // uniform row bases plus a 32-bit lane offset: no 64-bit address registers per load
      const char* xr = reinterpret_cast<const char*>(x + (int64_t)row * d);
      const char* rr = reinterpret_cast<const char*>(dres + (int64_t)row * d);
      const char* yr = reinterpret_cast<const char*>(dy + (int64_t)row * d);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        w.xh[q][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xr + cb[i]));
        w.rs[q][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(rr + cb[i]));
        w.dy[q][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(yr + (cb[i] >> 1)));
      }
    }
  };
  auto finish = [&](LnRows<NV, RF>& w, int row0, int k) {
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        w.xh[q][i] = (w.xh[q][i] - w.mu[q]) * w.r[q];
        const f32x4 dxh = bf16x4_to_f32(w.dy[q][i]) * gam[i];   // zero in columns past the end
        const f32x4 t = dxh * w.xh[q][i];
        s1 += (dxh.x + dxh.y) + (dxh.z + dxh.w);
        s2 += (t.x + t.y) + (t.z + t.w);
      }
      s1 = wave_sum_imm(s1); s2 = wave_sum_imm(s2);
      if (l == 0) { stat[k & 1][q][cs][0] = s1; stat[k & 1][q][cs][1] = s2; }
      // dy is widened again after the barrier rather than kept as fp32 across it (registers)
#pragma unroll
      for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(w.dy[q][i].x), "+v"(w.dy[q][i].y));
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < RF; ++q) {
      const int row = row0 + q;
      float s1 = stat[k & 1][q][0][0], s2 = stat[k & 1][q][0][1];
#pragma unroll
      for (int w2 = 1; w2 < CS; ++w2) { s1 += stat[k & 1][q][w2][0]; s2 += stat[k & 1][q][w2][1]; }
      const float c1 = s1 / (float)d, c2 = s2 / (float)d;
      if (row < T) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int c = cbase + 256 * i;
          if (c < d) {
            const f32x4 dyv = bf16x4_to_f32(w.dy[q][i]);
            const f32x4 dxh = dyv * gam[i];
            const f32x4 o = (dxh - c1 - w.xh[q][i] * c2) * w.r[q] + w.rs[q][i];
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(reinterpret_cast<char*>(dx + (int64_t)row * d) + cb[i]));
            if (dx_bf16)
              __builtin_nontemporal_store(f32_to_bf16x4(o), reinterpret_cast<u32x2*>(reinterpret_cast<char*>(dx_bf16 + (int64_t)row * d) + (cb[i] >> 1)));
            ag[i] += dyv * w.xh[q][i];
            ab[i] += dyv;
            ax[i] += o;
          }
          if (NV > 1) __builtin_amdgcn_sched_barrier(0);   // one column group's temporaries at a time
        }
      }
    }
  };
  const int rowb = blockIdx.x * ROWS;
  LnRows<NV, RF> wa, wb;
  request(wa, rowb);
#pragma unroll 1
  for (int k = 0; k < G - 2; k += 2) {
    request(wb, rowb + (k + 1) * RF);
    finish(wa, rowb + k * RF, k);
    request(wa, rowb + (k + 2) * RF);
    finish(wb, rowb + (k + 1) * RF, k + 1);
  }
  request(wb, rowb + (G - 1) * RF);
  finish(wa, rowb + (G - 2) * RF, G - 2);
  finish(wb, rowb + (G - 1) * RF, G - 1);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = cbase + 256 * i;
    if (c < d) {
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 0) * d + c) = ag[i];
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 1) * d + c) = ab[i];
      *reinterpret_cast<f32x4*>(part + ((int64_t)blockIdx.x * 3 + 2) * d + c) = ax[i];
    }
  }
}

// o = a widened to fp32, and the column sums of a over this workgroup's 32 rows as one partial
// row (the gradient arriving at the stage's output is also the bias gradient of its last Linear,
// summed over tokens).  A lane owns four columns.
constexpr int kWidenRows = 32;
__global__ __launch_bounds__(kThreads) void widen_colsum_kernel(const uint16_t* __restrict__ a, float* __restrict__ o,
                                                                float* __restrict__ part, int T, int d) {
  const int c = (blockIdx.x * kThreads + threadIdx.x) * 4;
  if (c >= d) return;
  const int r0 = blockIdx.y * kWidenRows;
  f32x4 acc = 0.f;
  static_assert(kWidenRows % 8 == 0, "batches of eight rows");
#pragma unroll 1
  for (int rb = r0; rb < r0 + kWidenRows; rb += 8) {
    u32x2 raw[8];                               // eight rows requested before the first is used
#pragma unroll
    for (int u = 0; u < 8; ++u) raw[u] = *reinterpret_cast<const u32x2*>(a + (int64_t)(rb + u < T ? rb + u : T - 1) * d + c);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (rb + u < T) {
        const f32x4 v = bf16x4_to_f32(raw[u]);
        *reinterpret_cast<f32x4*>(o + (int64_t)(rb + u) * d + c) = v;
        acc += v;
      }
  }
  *reinterpret_cast<f32x4*>(part + (int64_t)blockIdx.y * d + c) = acc;
}

// out_k[c] = sum_r src_k[r * pitch + c] for up to four (src, out) pairs in one launch
// (blockIdx.y picks the pair).  32 columns x 8 row lanes per workgroup; every row lane adds
// its rows in order, the eight partial sums are combined in a fixed order.
struct ReduceJobs {
  const float* src[4];
  float* out[4];      // null: the sums are not stored
  float* w[4];        // fp32 parameters updated in place with the sums (null: none), and
  uint16_t* ver[4];   // their bf16 weight version
  float eta;
};
__global__ __launch_bounds__(kThreads) void reduce_rows_kernel(ReduceJobs jobs, int R, int64_t pitch, int N) {
  __shared__ float red[8][33];
  const float* __restrict__ src = jobs.src[blockIdx.y];
  const int cl = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // eight loads in flight per lane
  if (c < N) {
    int r = rl;
    for (; r + 56 < R; r += 64) {
#pragma unroll
      for (int u = 0; u < 8; ++u) s[u] += src[(int64_t)(r + 8 * u) * pitch + c];
    }
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {       // the last, partial round: rows past the end re-read row R-1 and count as zero
      const int rr = r + 8 * u;
      t[u] = src[(int64_t)(rr < R ? rr : R - 1) * pitch + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) s[u] += r + 8 * u < R ? t[u] : 0.f;
  }
  red[rl][cl] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  if (rl == 0 && c < N) {
    float t = red[0][cl];
#pragma unroll
    for (int w = 1; w < 8; ++w) t += red[w][cl];
    if (jobs.out[blockIdx.y]) jobs.out[blockIdx.y][c] = t;
    if (jobs.w[blockIdx.y]) {   // delayed update of this small parameter vector (Eq. 2), where its gradient is born
      const float r = __fmaf_rn(-jobs.eta, t, jobs.w[blockIdx.y][c]);
      jobs.w[blockIdx.y][c] = r;
      jobs.ver[blockIdx.y][c] = rv_f32_to_bf16(r);
    }
  }
}

int nv_for(int d) { return d <= 1024 ? 4 : d <= 2048 ? 8 : d <= 4096 ? 16 : d <= 8192 ? 32 : 0; }

}  // namespace

rv_status rv_ln_fwd(const void* x, int x_is_bf16, float* xcopy, const uint16_t* gamma, const uint16_t* beta,
                    uint16_t* y, float* mean, float* rstd, int T, int d, float eps, hipStream_t st) {
  if (!x || !gamma || !beta || !y || !mean || !rstd || T < 1 || d < 4 || d % 4 || (x_is_bf16 && !xcopy))
    return RV_E_INVAL;
  const int nv = nv_for(d);
  if (!nv) return RV_E_INVAL;
  dim3 grid((T + kWaves - 1) / kWaves), blk(kThreads);
  if (!x_is_bf16 && d <= 1792) {
    const int rpw = T >= 8192 ? 4 : 2;
    dim3 g2((T + kWaves * rpw - 1) / (kWaves * rpw));
#define RV_LN_FWDP(NV, RPW) \
  hipLaunchKernelGGL((ln_fwd_pipe_kernel<NV, RPW>), g2, blk, 0, st, (const float*)x, gamma, beta, y, mean, rstd, T, d, eps);
    if (nv == 4) { if (rpw == 4) { RV_LN_FWDP(4, 4) } else { RV_LN_FWDP(4, 2) } }
    else { if (rpw == 4) { RV_LN_FWDP(7, 4) } else { RV_LN_FWDP(7, 2) } }
#undef RV_LN_FWDP
    return rv_launch_status();
  }
#define RV_LN_FWD(NV)                                                                                     \
  if (x_is_bf16)                                                                                          \
    hipLaunchKernelGGL((ln_fwd_kernel<NV, true>), grid, blk, 0, st, x, xcopy, gamma, beta, y, mean, rstd, T, d, eps); \
  else                                                                                                    \
    hipLaunchKernelGGL((ln_fwd_kernel<NV, false>), grid, blk, 0, st, x, xcopy, gamma, beta, y, mean, rstd, T, d, eps);
  switch (nv) {
    case 4: RV_LN_FWD(4) break;
    case 8: RV_LN_FWD(8) break;
    case 16: RV_LN_FWD(16) break;
    default: RV_LN_FWD(32) break;
  }
#undef RV_LN_FWD
  return rv_launch_status();
}

// Rows per workgroup: 8 for d <= 1024 (twice the workgroups: the stage step of the 1024-wide stage
// measured 0.4 % shorter than with 16, and 0.9 % shorter than with 4), 16 beyond (8 measured
// -0.2 % at d = 1600 and +0.2 % at d = 2048).
constexpr int kPipeRows = 8;
int rv_ln_bwd_parts(int T, int d) {
  const int rows = d <= 1024 ? kPipeRows : kRowsPerBlock;
  return (T + rows - 1) / rows;
}

rv_status rv_ln_bwd(const uint16_t* dy, const float* x, const float* mean, const float* rstd,
                    const uint16_t* gamma, const float* dres, float* dx, uint16_t* dx_bf16, float* part,
                    int T, int d, hipStream_t st) {
  if (!dy || !x || !mean || !rstd || !gamma || !dres || !dx || !part || T < 1 || d < 4 || d % 4 || d > 4096)
    return RV_E_INVAL;
  dim3 grid(rv_ln_bwd_parts(T, d)), blk(64 * kBwdWaves);
#define RV_LN_BWD(NV, RF) \
  hipLaunchKernelGGL((ln_bwd_kernel<NV, RF>), grid, blk, 0, st, dy, x, mean, rstd, gamma, dres, dx, dx_bf16, part, T, d);
  if (d <= 1024) {
    hipLaunchKernelGGL((ln_bwd_pipe_kernel<1, 2, kPipeRows>), grid, blk, 0, st, dy, x, mean, rstd, gamma, dres, dx, dx_bf16, part, T, d);
  }
  else if (d <= 2048) { RV_LN_BWD(2, 1) }
  else { RV_LN_BWD(4, 1) }
#undef RV_LN_BWD
  return rv_launch_status();
}

int rv_widen_parts(int T) { return (T + kWidenRows - 1) / kWidenRows; }

rv_status rv_widen_colsum(const uint16_t* a, float* o, float* part, int T, int d, hipStream_t st) {
  if (!a || !o || !part || T < 1 || d < 4 || d % 4) return RV_E_INVAL;
  dim3 grid((d / 4 + kThreads - 1) / kThreads, rv_widen_parts(T));
  hipLaunchKernelGGL(widen_colsum_kernel, grid, dim3(kThreads), 0, st, a, o, part, T, d);
  return rv_launch_status();
}

rv_status rv_reduce_rows_multi(const float* const* src, float* const* out, int njobs, int R, int64_t pitch,
                               int N, hipStream_t st, const rv_reduce_update* upd) {
  if (njobs < 1 || njobs > 4 || R < 1 || N < 1) return RV_E_INVAL;
  ReduceJobs j;
  j.eta = upd ? upd->eta : 0.f;
  for (int k = 0; k < 4; ++k) {
    j.src[k] = k < njobs ? src[k] : nullptr;
    j.out[k] = k < njobs && (!upd || upd->store) ? out[k] : nullptr;
    j.w[k] = k < njobs && upd ? upd->w[k] : nullptr;
    j.ver[k] = k < njobs && upd ? upd->ver[k] : nullptr;
    if (k < njobs && (!src[k] || !out[k] || (upd && (!upd->w[k] || !upd->ver[k])))) return RV_E_INVAL;
  }
  hipLaunchKernelGGL(reduce_rows_kernel, dim3((N + 31) / 32, njobs), dim3(kThreads), 0, st, j, R, pitch, N);
  return rv_launch_status();
}

rv_status rv_reduce_rows(const float* part, int R, int64_t pitch, int N, float* out, hipStream_t st,
                         const rv_reduce_update* upd) {
  return rv_reduce_rows_multi(&part, &out, 1, R, pitch, N, st, upd);
}

extern "C" rv_status rv_k_layernorm_fwd(const void* x, int x_is_bf16, float* xcopy, const void* gamma,
                                        const void* beta, void* y, float* mean, float* rstd, int T, int d,
                                        float eps, void* stream) {
  return rv_ln_fwd(x, x_is_bf16, xcopy, (const uint16_t*)gamma, (const uint16_t*)beta, (uint16_t*)y, mean, rstd,
                   T, d, eps, (hipStream_t)stream);
}

extern "C" rv_status rv_k_layernorm_bwd(const void* dy, const float* x, const float* mean, const float* rstd,
                                        const void* gamma, const float* dres, float* dx, void* dx_bf16,
                                        float* part, float* dgamma, float* dbeta, float* dbias, int T, int d,
                                        void* stream) {
  hipStream_t st = (hipStream_t)stream;
  RV_TRY(rv_ln_bwd((const uint16_t*)dy, x, mean, rstd, (const uint16_t*)gamma, dres, dx, (uint16_t*)dx_bf16,
                   part, T, d, st));
  const int R = rv_ln_bwd_parts(T, d);
  const float* src[3]; float* out[3]; int n = 0;
  if (dgamma) { src[n] = part; out[n++] = dgamma; }
  if (dbeta) { src[n] = part + d; out[n++] = dbeta; }
  if (dbias) { src[n] = part + 2 * d; out[n++] = dbias; }
  return n ? rv_reduce_rows_multi(src, out, n, R, 3 * (int64_t)d, d, st) : RV_OK;
}
