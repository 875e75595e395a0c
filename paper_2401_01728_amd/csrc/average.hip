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
// Layout: one workgroup owns a tile of TILE consecutive elements.  Chunks are millions of
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
constexpr int kVecPerThread = 1;                       // float4 per lane
constexpr int kTile = kThreads * kVecPerThread * 4;    // elements per tile

// Owning chunk of element i: ring r = ceil((i+1) R / n) - 1, then the same rule inside
// the ring's segment.
__device__ __forceinline__ int chunk_of(uint64_t i, uint64_t n, int R, int C) {
  uint64_t r = ((i + 1) * (uint64_t)R - 1) / n;
  uint64_t lo = (r * n) / (uint64_t)R;
  uint64_t hi = ((r + 1) * n) / (uint64_t)R;
  uint64_t s = hi - lo;
  return (int)(((i - lo + 1) * (uint64_t)C - 1) / s);
}

// Rings given by explicit boundaries (segments of unequal size, as when clusters split the
// model differently and a peer sits in several rings): off[0] = 0 <= ... <= off[R] = n.
#define RV_MAX_EXPLICIT_R 64
struct RingOffsets {
  uint64_t off[RV_MAX_EXPLICIT_R + 1];
};
__device__ __forceinline__ void ring_of(const RingOffsets& ro, int R, uint64_t i, uint64_t& lo, uint64_t& hi) {
  int r = 0;
  while (r + 1 < R && i >= ro.off[r + 1]) ++r;     // empty rings are stepped over
  lo = ro.off[r]; hi = ro.off[r + 1];
}
__device__ __forceinline__ int chunk_of_v(const RingOffsets& ro, int R, uint64_t i, int C) {
  uint64_t lo, hi;
  ring_of(ro, R, i, lo, hi);
  return (int)(((i - lo + 1) * (uint64_t)C - 1) / (hi - lo));
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

// The C replica base pointers are fetched with scalar loads in ring order starting at j
// (wave-uniform), every lane issues its C independent 16-byte loads, then adds them in
// that order.  (A compile-time rotation of the SUM order over naturally ordered loads was
// tried: the compiler folds the C unrolled variants back into a dynamically indexed
// register array in scratch memory, which costs a third of the bandwidth.)
template <int C, bool HAS_GRAD>
__device__ __forceinline__ void tile_fast(const RepTable& tab, int j, uint64_t base, float* out,
                                          int write_back, const float* grad, int gr, float eta) {
  const float c_num = (float)C;
  j = __builtin_amdgcn_readfirstlane(j);
#pragma unroll
  for (int u = 0; u < kVecPerThread; ++u) {
    const uint64_t e = base + (uint64_t)(u * kThreads + threadIdx.x) * 4;
    f4 v[C];
#pragma unroll
    for (int s = 0; s < C; ++s) {
      int c = j + s; if (c >= C) c -= C;
      v[s] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(tab.p[c] + e));
      if (HAS_GRAD && c == gr) {
        const f4 g = __builtin_nontemporal_load(reinterpret_cast<const f4*>(grad + e));
        v[s].x = __fsub_rn(v[s].x, __fmul_rn(g.x, eta));
        v[s].y = __fsub_rn(v[s].y, __fmul_rn(g.y, eta));
        v[s].z = __fsub_rn(v[s].z, __fmul_rn(g.z, eta));
        v[s].w = __fsub_rn(v[s].w, __fmul_rn(g.w, eta));
      }
    }
    f4 a = v[0];
#pragma unroll
    for (int s = 1; s < C; ++s) {
      a.x = __fadd_rn(a.x, v[s].x); a.y = __fadd_rn(a.y, v[s].y);
      a.z = __fadd_rn(a.z, v[s].z); a.w = __fadd_rn(a.w, v[s].w);
    }
    a.x = __fdiv_rn(a.x, c_num);
    a.y = __fdiv_rn(a.y, c_num);
    a.z = __fdiv_rn(a.z, c_num);
    a.w = __fdiv_rn(a.w, c_num);
    if (out != nullptr) __builtin_nontemporal_store(a, reinterpret_cast<f4*>(out + e));
    if (write_back) {
#pragma unroll
      for (int c = 0; c < C; ++c)
        __builtin_nontemporal_store(a, reinterpret_cast<f4*>(tab.p[c] + e));
    }
  }
}

// floor(x / d) for x < 2^52 from an fp64 estimate (inv_d = 1/d rounded) and one exact
// correction step: the estimate is within one of the quotient, q*d fits in 64 bits.
__device__ __forceinline__ uint64_t floor_div(uint64_t x, uint64_t d, double inv_d) {
  uint64_t q = (uint64_t)((double)x * inv_d);
  if (q * d > x) --q;
  else if ((q + 1) * d <= x) ++q;
  return q;
}

struct DivConsts {
  double inv_n, inv_R, inv_C;
};

// Chunk that owns element i and the (exclusive) end of that chunk: the same arithmetic as
// chunk_of, without 64-bit integer division (it runs once per workgroup).
__device__ __forceinline__ void locate(uint64_t i, uint64_t n, int R, int C, const DivConsts& dc, int& j,
                                       uint64_t& chunk_end) {
  const uint64_t r = floor_div((i + 1) * (uint64_t)R - 1, n, dc.inv_n);
  const uint64_t lo = floor_div(r * n, (uint64_t)R, dc.inv_R), hi = floor_div((r + 1) * n, (uint64_t)R, dc.inv_R);
  const uint64_t s = hi - lo;
  j = (int)floor_div((i - lo + 1) * (uint64_t)C - 1, s, 1.0 / (double)s);
  chunk_end = lo + floor_div((uint64_t)(j + 1) * s, (uint64_t)C, dc.inv_C);
}

// One workgroup per tile.  C == 0 instantiates the generic (runtime-C) kernel, which only
// has the element path.
template <int CT, bool HAS_GRAD, bool EXPL>
__global__ __launch_bounds__(kThreads) void average_kernel(RepTable tab, int Crt, uint64_t n, int R,
                                                           float* out, int write_back,
                                                           const float* grad, int gr, float eta,
                                                           int aligned, DivConsts dc, RingOffsets ro) {
  const int C = CT > 0 ? CT : Crt;
  const uint64_t base = (uint64_t)blockIdx.x * kTile, last = base + kTile - 1;
  if constexpr (CT > 0) {
    if (aligned) {
      int j;
      uint64_t chunk_end;
      if (EXPL) {
        uint64_t lo, hi;
        ring_of(ro, R, base, lo, hi);
        const uint64_t sz = hi - lo;
        j = (int)floor_div((base - lo + 1) * (uint64_t)C - 1, sz, 1.0 / (double)sz);
        chunk_end = lo + floor_div((uint64_t)(j + 1) * sz, (uint64_t)C, dc.inv_C);
      } else {
        locate(base, n, R, C, dc, j, chunk_end);   // wave-uniform, no barrier needed
      }
      if (last < chunk_end) {                    // chunk_end <= n: the tile is whole and inside one chunk
        tile_fast<CT, HAS_GRAD>(tab, j, base, out, write_back, grad, gr, eta);
        return;
      }
    }
  }
  for (int k = threadIdx.x; k < kTile; k += kThreads) {
    const uint64_t i = base + k;
    if (i >= n) break;
    const int je = EXPL ? chunk_of_v(ro, R, i, C) : chunk_of(i, n, R, C);
    const float m = elem_mean(tab, C, je, i, HAS_GRAD ? grad : nullptr, gr, eta);
    if (out != nullptr) out[i] = m;
    if (write_back)
      for (int c = 0; c < C; ++c) tab.p[c][i] = m;
  }
}

template <int CT>
void launch(const RepTable& tab, int C, uint64_t n, int R, float* out, int wb, const float* grad,
            int gr, float eta, int aligned, const RingOffsets* ro, hipStream_t st) {
  const unsigned blocks = (unsigned)((n + kTile - 1) / kTile);
  const DivConsts dc{1.0 / (double)n, 1.0 / (double)R, 1.0 / (double)C};
  static const RingOffsets none = {};
#define RV_AVG_LAUNCH(G, E)                                                                              \
  hipLaunchKernelGGL((average_kernel<CT, G, E>), dim3(blocks), dim3(kThreads), 0, st, tab, C, n, R, out, \
                     wb, grad, gr, eta, aligned, dc, E ? *ro : none)
  if (ro) { if (grad) RV_AVG_LAUNCH(true, true); else RV_AVG_LAUNCH(false, true); }
  else    { if (grad) RV_AVG_LAUNCH(true, false); else RV_AVG_LAUNCH(false, false); }
#undef RV_AVG_LAUNCH
}

}  // namespace

static rv_status average_impl(float* const* replicas, int C, size_t n, int R, const RingOffsets* ro,
                              float* mean_out, int write_back, const float* grad, int grad_replica, float eta,
                              void* stream) {
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
    case 1: launch<1>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    case 2: launch<2>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    case 3: launch<3>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    case 4: launch<4>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    case 8: launch<8>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    case 16: launch<16>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
    default: launch<0>(tab, C, n, R, mean_out, wb, grad, grad_replica, eta, aligned, ro, st); break;
  }
  return rv_launch_status();
}

extern "C" rv_status rv_cluster_average(float* const* replicas, int C, size_t n, int R,
                                        float* mean_out, int write_back, const float* grad,
                                        int grad_replica, float eta, void* stream) {
  return average_impl(replicas, C, n, R, nullptr, mean_out, write_back, grad, grad_replica, eta, stream);
}

extern "C" rv_status rv_cluster_average_v(float* const* replicas, int C, size_t n, const int64_t* ring_offsets,
                                          int R, float* mean_out, int write_back, const float* grad,
                                          int grad_replica, float eta, void* stream) {
  if (ring_offsets == nullptr || R < 1 || R > RV_MAX_EXPLICIT_R) return RV_E_INVAL;
  if (ring_offsets[0] != 0 || ring_offsets[R] != (int64_t)n) return RV_E_INVAL;
  RingOffsets ro = {};
  for (int r = 0; r <= R; ++r) {
    if (r > 0 && ring_offsets[r] < ring_offsets[r - 1]) return RV_E_INVAL;
    ro.off[r] = (uint64_t)ring_offsets[r];
  }
  return average_impl(replicas, C, n, R, &ro, mean_out, write_back, grad, grad_replica, eta, stream);
}
