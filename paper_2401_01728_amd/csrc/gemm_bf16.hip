// bf16 MFMA matrix products of the decoder stage (forward, dX and dW of every Linear),
// fp32 accumulation, for gfx950.
//
//   C[M,N] = sum_k A(m,k) B(k,n)        K % 64 == 0, N % 8 == 0, M % 8 == 0
//
// Each operand is either "k-contiguous" (A[m*lda+k], B[n*ldb+k]) or "k-major"
// (A[k*lda+m], B[k*ldb+n]).  The three products of a Linear y = x W, W stored [in,out]:
//   forward  y  = x W      : A = x  k-contiguous, B = W  k-major
//   dX       dx = dy W^T   : A = dy k-contiguous, B = W  k-contiguous (its rows are the n's)
//   dW       dW = x^T dy   : A = x  k-major,      B = dy k-major      (contraction over tokens)
//
// Tiling: a workgroup of 4 or 8 waves owns a BM x BN tile and walks K in steps of BK (32 or
// 64); a wave owns a block of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16).  Operand tiles go
// global -> LDS directly (global_load_lds_dwordx4) through a ring of NS stages, unpadded, bank
// conflicts removed by an XOR swizzle (see "direct-to-LDS pipeline" below);
//   k-contiguous operands sit in LDS as [row][BK k], read as one 16-byte fragment per lane;
//   k-major operands sit as [BK k][cols] and are read with the LDS transpose read
//   (ds_read_b64_tr_b16), which hands each lane four consecutive k of one column: no register
//   transposes, no transposed copies of activations in HBM.
// The MFMA is issued with the B fragment as its first operand, so a lane ends up with
// four CONSECUTIVE n of one row m: epilogues store 8 (bf16) or 16 (fp32) bytes per lane.
#include "internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// GELU(z) = z * Phi(z) and its derivative Phi(z) + z * phi(z).  The upper tail of the normal
// distribution, q = 1 - Phi(|z|) = erfc(|z|/sqrt 2)/2, comes from the three-term
// rational-exponential form of erfc (Abramowitz & Stegun 7.1.25, |error| < 1.3e-5 on q - the
// results are rounded to bf16, whose half-ulp is 2e-3 relative):
//   q = (a1 t + a2 t^2 + a3 t^3)/2 * exp(-z^2/2),   t = 1/(1 + 0.47047 |z|/sqrt 2).
// Computing the tail directly loses no digits to cancellation for negative arguments, and
//   GELU(z) = max(z, 0) - |z| q
// needs no select.  The same exponential serves phi(z).  Nine instructions, two of them
// transcendental.
__device__ __forceinline__ float tail_q(float z, float& e) {
  const float t = __builtin_amdgcn_rcpf(__fmaf_rn(fabsf(z), 0.33267254f, 1.0f));
  e = __builtin_amdgcn_exp2f(z * z * -0.72134752f);
  float p = __fmaf_rn(0.3739278f, t, -0.0479399f);
  p = __fmaf_rn(p, t, 0.1740121f);
  return p * t * e;
}
__device__ __forceinline__ float gelu_f(float z) {
  float e;
  const float q = tail_q(z, e);
  return __fmaf_rn(-fabsf(z), q, fmaxf(z, 0.f));
}
__device__ __forceinline__ float dgelu_f(float z) {
  float e;
  const float q = tail_q(z, e);
  const float cdf = z < 0.f ? q : 1.0f - q;
  return __fmaf_rn(z * 0.3989422804014327f, e, cdf);
}

#ifndef RV_RESID_LDS
#define RV_RESID_LDS 1
#endif
struct Epi {
  void* out; int64_t ldo;
  void* out2;
  const uint16_t* bias;
  const float* resid; int64_t ldr;
  const uint16_t* zin;
  float* upd_w;   // EPI_F32_UPD: fp32 master tile updated in place (out2 = its bf16 weight version)
  float eta;
  float* colpart; // EPI_BF16_DGELU: partial column sums of the output, one row (pitch ldo) per tile row
};

enum { EPI_BF16 = RV_EPI_BF16, EPI_BF16_BIAS = RV_EPI_BF16_BIAS, EPI_F32_BIAS_RESID = RV_EPI_F32_BIAS_RESID,
       EPI_BF16_BIAS_GELU = RV_EPI_BF16_BIAS_GELU, EPI_BF16_DGELU = RV_EPI_BF16_DGELU, EPI_F32 = RV_EPI_F32,
       EPI_F32_BIAS_RESID_BF16 = RV_EPI_F32_BIAS_RESID_BF16,
       // grouped weight-gradient launch only: out f32 = acc if out is given; if upd_w is given the
       // delayed update of Eq. 2 right here, w <- w - eta * acc (one fused multiply-add, as the
       // stand-alone update kernel does it) and out2 bf16 = the new w
       EPI_F32_UPD = 7 };

constexpr bool epi_has_bias(int epi) {
  return epi == EPI_BF16_BIAS || epi == EPI_F32_BIAS_RESID || epi == EPI_BF16_BIAS_GELU || epi == EPI_F32_BIAS_RESID_BF16;
}
constexpr bool epi_has_resid(int epi) { return epi == EPI_F32_BIAS_RESID || epi == EPI_F32_BIAS_RESID_BF16; }

__device__ __forceinline__ void add_bias4(f32x4& a, u32x2 b) {
  a.x += __uint_as_float(b.x << 16); a.y += __uint_as_float(b.x & 0xFFFF0000u);
  a.z += __uint_as_float(b.y << 16); a.w += __uint_as_float(b.y & 0xFFFF0000u);
}

// four consecutive columns n..n+3 of row m; b = their bias, r = their residual (already loaded)
template <int EPI>
__device__ __forceinline__ void epilogue4(const Epi& e, int m, int n, f32x4 a, u32x2 b, f32x4 r) {
  if (epi_has_bias(EPI)) add_bias4(a, b);
  if (EPI == EPI_BF16 || EPI == EPI_BF16_BIAS) {
    u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
    *reinterpret_cast<u32x2*>((uint16_t*)e.out + (int64_t)m * e.ldo + n) = o;
  } else if (epi_has_resid(EPI)) {
    a += r;
    *reinterpret_cast<f32x4*>((float*)e.out + (int64_t)m * e.ldo + n) = a;
    if (EPI == EPI_F32_BIAS_RESID_BF16) {
      u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
      *reinterpret_cast<u32x2*>((uint16_t*)e.out2 + (int64_t)m * e.ldo + n) = o;
    }
  } else if (EPI == EPI_BF16_BIAS_GELU) {
    u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
    *reinterpret_cast<u32x2*>((uint16_t*)e.out + (int64_t)m * e.ldo + n) = o;
    u32x2 g;
    g.x = rv_pack_bf16x2(gelu_f(a.x), gelu_f(a.y));
    g.y = rv_pack_bf16x2(gelu_f(a.z), gelu_f(a.w));
    *reinterpret_cast<u32x2*>((uint16_t*)e.out2 + (int64_t)m * e.ldo + n) = g;
  } else if (EPI == EPI_BF16_DGELU) {
    u32x2 z = *reinterpret_cast<const u32x2*>(e.zin + (int64_t)m * e.ldo + n);
    a.x *= dgelu_f(__uint_as_float(z.x << 16)); a.y *= dgelu_f(__uint_as_float(z.x & 0xFFFF0000u));
    a.z *= dgelu_f(__uint_as_float(z.y << 16)); a.w *= dgelu_f(__uint_as_float(z.y & 0xFFFF0000u));
    u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
    *reinterpret_cast<u32x2*>((uint16_t*)e.out + (int64_t)m * e.ldo + n) = o;
  } else if (EPI == EPI_F32) {
    *reinterpret_cast<f32x4*>((float*)e.out + (int64_t)m * e.ldo + n) = a;
  } else if (EPI == EPI_F32_UPD) {
    // (no update asked for: the gradient tile alone; the update path is f32_tile_through_lds)
    *reinterpret_cast<f32x4*>((float*)e.out + (int64_t)m * e.ldo + n) = a;
  }
}

// lane holds row m = l%32 of the wave tile and, per group rg of 4 registers,
// columns 8*rg + 4*(l/32) .. +3
// What an epilogue reads (bias, residual) is requested for a whole batch of column groups, at
// addresses clamped into the matrix, before the first result is formed: a batch costs one
// memory round trip, not one per group of four columns.
template <int TM, int TN, int EPI>
__device__ __forceinline__ void write_tile(const f32x16 (&acc)[TM][TN], const Epi& e, int mw, int nw, int M, int N) {
  const int l = threadIdx.x & 63;
  constexpr int JB = TN > 2 ? 2 : TN;          // tile columns per batch of residual loads
  u32x2 bias4[TN][4];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      bias4[j][rg] = u32x2{0u, 0u};
      if (epi_has_bias(EPI)) {
        const int n = nw + j * 32 + 8 * rg + 4 * (l >> 5);
        bias4[j][rg] = *reinterpret_cast<const u32x2*>(e.bias + (n < N ? n : N - 4));
      }
    }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = mw + i * 32 + (l & 31);
    const int mc = m < M ? m : M - 1;
#pragma unroll
    for (int j0 = 0; j0 < TN; j0 += JB) {
      f32x4 res[JB][4];
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          res[jj][rg] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (epi_has_resid(EPI)) {
            const int n = nw + (j0 + jj) * 32 + 8 * rg + 4 * (l >> 5);
            res[jj][rg] = *reinterpret_cast<const f32x4*>(e.resid + (int64_t)mc * e.ldr + (n < N ? n : N - 4));
          }
        }
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int j = j0 + jj;
          const int n = nw + j * 32 + 8 * rg + 4 * (l >> 5);
          if (m >= M || n >= N) continue;
          f32x4 a = {acc[i][j][4 * rg], acc[i][j][4 * rg + 1], acc[i][j][4 * rg + 2], acc[i][j][4 * rg + 3]};
          epilogue4<EPI>(e, m, n, a, bias4[j][rg], res[jj][rg]);
        }
    }
  }
}

// Workgroup -> tile map (tiles_m > 0; a negative tiles_m selects the natural order).
// Workgroups are dealt to the 8 XCDs round-robin (id % 8), and each
// XCD has its own L2.  First give every XCD a CONTIGUOUS range of tile numbers, then walk
// that range in bands of 8 tile-rows, column by column: the ~32 tiles an XCD has in flight
// form an 8 x 4 patch, so it pulls 12 operand tiles per k-step through its L2 instead of 33.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int band_rows, int& bm, int& bn) {
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  if (tiles_m < 0) {   // natural order: consecutive workgroups walk down one column of tiles
    tiles_m = -tiles_m; bm = id % tiles_m; bn = id / tiles_m; return;
  }
  const int per = total / 8;
  if (id < per * 8) id = (id % 8) * per + id / 8;       // the remainder keeps its natural order
  const int GM = band_rows;
  const int band = id / (GM * tiles_n);
  const int first = band * GM;
  const int rows = tiles_m - first < GM ? tiles_m - first : GM;
  const int in = id - band * GM * tiles_n;
  bm = first + in % rows;
  bn = in / rows;
}

// bf16 outputs leave through LDS: every wave parks its accumulator tile (after bias / GELU /
// GELU') as bf16 in a [BM][BN] image of the workgroup tile, then the workgroup writes the
// image out row by row, 16 bytes per lane, whole 128-byte lines per row segment - instead
// of 8-byte pieces of 32 different rows per store instruction.  The GELU epilogue makes two
// trips (pre-activation, then activation).  The image reuses the operand ring.
__host__ __device__ constexpr int stage_pitch(int bn) { return bn * 2 + 16; }
__host__ __device__ constexpr bool staged_epi(int epi) {
  return epi == EPI_BF16 || epi == EPI_BF16_BIAS || epi == EPI_BF16_BIAS_GELU || epi == EPI_BF16_DGELU;
}

template <int BM, int BN, int NT, int TM, int TN, int EPI>
__device__ __forceinline__ void write_tile_staged(const f32x16 (&acc)[TM][TN], const Epi& e, int m0, int n0,
                                                  int wm0, int wn0, int M, int N, char* smem) {
  constexpr int PITCH = stage_pitch(BN);
  constexpr int PASSES = EPI == EPI_BF16_BIAS_GELU ? 2 : 1;
  const int l = threadIdx.x & 63;
  __syncthreads();   // every wave has finished reading operands from the ring
  if (EPI == EPI_BF16_DGELU) {
    // the pre-activation tile comes in the way the result goes out: whole rows, 16 bytes per
    // lane, through the image; a lane then finds its own four values where it will put the result
    // (eight loads per lane in flight before the first is parked: two memory round trips per
    // tile instead of one per 16-byte piece)
    constexpr int CPR = BN / 8, PIECES = BM * CPR / NT, BATCH = NT >= 512 ? 8 : 4;
    static_assert(BM * CPR % NT == 0 && PIECES % BATCH == 0, "whole batches");
#pragma unroll 1
    for (int p0 = 0; p0 < PIECES; p0 += BATCH) {
      u32x4 v[BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int idx = threadIdx.x + (p0 + u) * NT, row = idx / CPR, c = idx % CPR;
        const int gm = m0 + row, gn = n0 + c * 8;
        v[u] = u32x4{0u, 0u, 0u, 0u};
        if (gm < M && gn < N) v[u] = *reinterpret_cast<const u32x4*>(e.zin + (int64_t)gm * e.ldo + gn);
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int idx = threadIdx.x + (p0 + u) * NT, row = idx / CPR, c = idx % CPR;
        *reinterpret_cast<u32x4*>(smem + row * PITCH + c * 16) = v[u];
      }
    }
    __syncthreads();
  }
  // GELU' epilogue: column sums of the results over this wave's rows, kept per lane while the tile
  // is packed (the bias gradient of the Linear below the GELU, one partial row per tile row)
  f32x4 cs[TN][4];
  const bool want_cs = EPI == EPI_BF16_DGELU && e.colpart != nullptr;
  float* red = reinterpret_cast<float*>(smem + BM * PITCH);   // [2 wave rows][BN], behind the image
  if (EPI == EPI_BF16_DGELU) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) cs[j][rg] = 0.f;
  }
  u32x2 bias4[TN][4];                            // this lane's bias values, loaded once
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      bias4[j][rg] = u32x2{0u, 0u};
      if (EPI == EPI_BF16_BIAS || EPI == EPI_BF16_BIAS_GELU) {
        const int gn = n0 + wn0 + j * 32 + 8 * rg + 4 * (l >> 5);
        bias4[j][rg] = *reinterpret_cast<const u32x2*>(e.bias + (gn < N ? gn : N - 4));
      }
    }
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int ml = wm0 + i * 32 + (l & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int nl = wn0 + j * 32 + 8 * rg + 4 * (l >> 5);
          const int gm = m0 + ml, gn = n0 + nl;
          f32x4 a = {acc[i][j][4 * rg], acc[i][j][4 * rg + 1], acc[i][j][4 * rg + 2], acc[i][j][4 * rg + 3]};
          if (EPI == EPI_BF16_BIAS || EPI == EPI_BF16_BIAS_GELU) {
            add_bias4(a, bias4[j][rg]);
            if (pass == 1) { a.x = gelu_f(a.x); a.y = gelu_f(a.y); a.z = gelu_f(a.z); a.w = gelu_f(a.w); }
          }
          if (EPI == EPI_BF16_DGELU) {
            if (gm < M && gn < N) {
              const u32x2 z = *reinterpret_cast<const u32x2*>(smem + ml * PITCH + nl * 2);
              a.x *= dgelu_f(__uint_as_float(z.x << 16)); a.y *= dgelu_f(__uint_as_float(z.x & 0xFFFF0000u));
              a.z *= dgelu_f(__uint_as_float(z.y << 16)); a.w *= dgelu_f(__uint_as_float(z.y & 0xFFFF0000u));
              cs[j][rg] += a;
            }
          }
          u32x2 o; o.x = rv_pack_bf16x2(a.x, a.y); o.y = rv_pack_bf16x2(a.z, a.w);
          *reinterpret_cast<u32x2*>(smem + ml * PITCH + nl * 2) = o;
        }
      }
    }
    if (EPI == EPI_BF16_DGELU && want_cs) {   // (workgroup-uniform)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          f32x4 v;
          v.x = rv_half_wave_sum(cs[j][rg].x); v.y = rv_half_wave_sum(cs[j][rg].y);
          v.z = rv_half_wave_sum(cs[j][rg].z); v.w = rv_half_wave_sum(cs[j][rg].w);
          if ((l & 31) == 0)
            *reinterpret_cast<f32x4*>(red + (wm0 ? BN : 0) + wn0 + j * 32 + 8 * rg + 4 * (l >> 5)) = v;
        }
    }
    __syncthreads();
    if (EPI == EPI_BF16_DGELU && want_cs) {
      for (int c = threadIdx.x; c < BN; c += NT)
        if (n0 + c < N) e.colpart[(int64_t)(m0 / BM) * e.ldo + n0 + c] = red[c] + red[BN + c];
    }
    uint16_t* dst = (uint16_t*)(pass == 0 ? e.out : e.out2);
    constexpr int CPR = BN / 8, PIECES = BM * CPR / NT, BATCH = NT >= 512 ? 8 : 4;
    static_assert(BM * CPR % NT == 0 && PIECES % BATCH == 0, "whole batches");
#pragma unroll 1
    for (int p0 = 0; p0 < PIECES; p0 += BATCH) {
      u32x4 v[BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int idx = threadIdx.x + (p0 + u) * NT, row = idx / CPR, c = idx % CPR;
        v[u] = *reinterpret_cast<const u32x4*>(smem + row * PITCH + c * 16);
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int idx = threadIdx.x + (p0 + u) * NT, row = idx / CPR, c = idx % CPR;
        const int gm = m0 + row, gn = n0 + c * 8;
        if (gm < M && gn < N) *reinterpret_cast<u32x4*>(dst + (int64_t)gm * e.ldo + gn) = v[u];
      }
    }
    if (pass + 1 < PASSES) __syncthreads();
  }
}

// ---- direct-to-LDS pipeline ---------------------------------------------------------------
// Tiles go global -> LDS with global_load_lds_dwordx4: no staging registers, no LDS write
// instructions.  One such instruction fills 1 KiB of LDS (lane i -> base + 16 i), so the
// tile is unpadded and bank conflicts are removed by an XOR swizzle of the 16-byte chunk
// index instead; because a lane's LDS slot is fixed, the swizzle is applied to the GLOBAL
// address a lane fetches.
//   k-contiguous tile [rows][BK]: physical chunk = c ^ ((row / rows_per_256B) % chunks_per_row)
//   k-major tile [BK][cols]     : physical chunk = c ^ ((k & 3) << 2)   (64-byte granules)
// NS stages form a ring.  Plain form (four-wave tiles): the loads of tile t+NS-1 are issued
// right after the barrier that opens tile t.  Pipelined form (the eight-wave 256x256 tile): see
// gemm_dtl_body - the products are bound by how fast operand tiles arrive, inside a stage step
// even more than alone (with seven of eight MFMAs taken out the step is 3 % shorter, without
// the loads 24 %), so that tile keeps three 32-deep tiles in flight instead of one 64-deep one.
__host__ __device__ constexpr int dtl_tile_bytes(int rows, int bk) { return rows * bk * 2; }

template <bool KM, int ROWS, int BK, int NW>
struct Dtl {
  static constexpr int N = ROWS * BK / 8 / (64 * NW);   // loads per lane per tile
  int off[N];
};

template <bool KM, int ROWS, int BK, int NW>
__device__ __forceinline__ void dtl_init(Dtl<KM, ROWS, BK, NW>& s, int64_t ld, int r0, int rows, int wave) {
  const int l = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < Dtl<KM, ROWS, BK, NW>::N; ++i) {
    const int slot = (i * NW + wave) * 64 + l;
    if (!KM) {
      constexpr int CPR = BK / 8, R256 = 256 / (BK * 2);
      const int row = slot / CPR, c = (slot % CPR) ^ ((row / R256) % CPR);
      int gr = r0 + row;
      gr = gr < rows ? gr : rows - 1;
      s.off[i] = gr * (int)ld + c * 8;
    } else {
      constexpr int CPR = ROWS / 8;
      const int kr = slot / CPR, c = (slot % CPR) ^ ((kr & 3) << 2);
      int col = r0 + c * 8;
      col = col < rows ? col : rows - 8;
      s.off[i] = kr * (int)ld + col;
    }
  }
}

template <bool KM, int ROWS, int BK, int NW>
__device__ __forceinline__ void dtl_issue(const Dtl<KM, ROWS, BK, NW>& s, const uint16_t* __restrict__ g,
                                          int64_t ld, int k0, char* lds, int wave) {
  const uint16_t* base = KM ? g + (int64_t)k0 * ld : g + k0;
#pragma unroll
  for (int i = 0; i < Dtl<KM, ROWS, BK, NW>::N; ++i) {
    // LDS byte address of this wave's 1 KiB block (wave-uniform, goes to M0; the hardware
    // adds 16 * lane).  Issued as inline assembly: the compiler would otherwise make every
    // later LDS read wait for ALL outstanding loads, which defeats the ring.  The kernel
    // orders them itself with explicit vmcnt waits and barriers.
    const int m0v = __builtin_amdgcn_readfirstlane((int)(size_t)lds + (i * NW + wave) * 1024);
    const uint16_t* src = base + s.off[i];
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(m0v)
                 : "memory", "m0");
  }
}

template <bool KM, int ROWS, int BK>
__device__ __forceinline__ bf16x8 dtl_frag(const char* lds, int row0, int kk) {
  const int l = threadIdx.x & 63;
  if (!KM) {
    constexpr int CPR = BK / 8, R256 = 256 / (BK * 2);
    const int row = row0 + (l & 31);
    const int c = (kk * 2 + (l >> 5)) ^ ((row / R256) % CPR);
    return *reinterpret_cast<const bf16x8*>(lds + row * (BK * 2) + c * 16);
  } else {
    const int q = l >> 4, i = l & 15;
    const int kr = kk * 16 + 8 * (q >> 1) + (i >> 2);
    const int col = row0 + 16 * (q & 1) + 4 * (i & 3);
    const int c = (col >> 3) ^ ((kr & 3) << 2);
    const char* p = lds + kr * (ROWS * 2) + c * 16 + (col & 7) * 2;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(p + 4 * (ROWS * 2)));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
  }
}

// Direct-to-LDS load in the scalar-base form: wave-uniform 64-bit base in SGPRs, per-lane byte
// offset in one VGPR (no per-load address arithmetic), LDS block = lb + IMM through M0.
__device__ __forceinline__ void dtl_load_s(const void* base, unsigned off, int m0v) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(base), "s"(m0v)
               : "memory", "m0");
}
// s_waitcnt vmcnt(n) only (expcnt, lgkmcnt left at "no wait"); n < 64
#define RV_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

extern __shared__ __align__(1024) char dtl_smem[];

// Epilogue of a weight-gradient tile with the delayed update of Eq. 2 folded in:
//   w <- w - eta * acc (fp32 master, in place), bf16(w) into the new weight version, acc itself
// to `out` only on request.  The master tile is fetched through LDS, half a tile at a time,
// with direct-to-LDS loads (one instruction = one 256-column fp32 row): all rows of the half
// are in flight together, so the read costs one memory round trip per half instead of one per
// accumulator group, and it needs no registers.  Row pitch BN*4 + 16 bytes spreads a wave's
// 32 rows over the banks.
__host__ __device__ constexpr int upd_image_bytes(int bm, int bn) { return (bm / 2) * (bn * 4 + 16); }

// MODE 0: the update above (source and fp32 result = e.upd_w, bf16 result = e.out2, the gradient itself to e.out
//         on request).  MODE 1: out = acc + bias + residual (source = e.resid, fp32 result = e.out, and with
//         BF16OUT its rounding to e.out2) - the same staging: at 4-byte results per lane-quad the direct form costs
//         more L2 requests than a short product's whole main loop.
// The results go back into the LDS rows they came from and leave the way the rows came in: whole rows, 16 bytes
// per lane, one 128-byte line per 8 lanes, instead of 32-byte pieces of 32 different rows per store instruction.
template <int BM, int BN, int NW, int TM, int TN, int MODE, bool BF16OUT>
__device__ __forceinline__ void f32_tile_through_lds(const f32x16 (&acc)[TM][TN], const Epi& e, int m0, int n0,
                                                     int wm0, int wn0, int M, int N, char* smem) {
  static_assert(BN == 256, "one direct-to-LDS instruction moves one 256-column fp32 row");
  constexpr int HALF = BM / 2, PITCH = BN * 4 + 16, RPW = HALF / NW;   // rows per wave in the row-wise phases
  static_assert(HALF % NW == 0 && RPW % 8 == 0, "row batches of eight");
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  const float* srcm = MODE == 0 ? e.upd_w : e.resid;
  const int64_t lds_src = MODE == 0 ? e.ldo : e.ldr;
  float* dst32 = MODE == 0 ? e.upd_w : (float*)e.out;
  u32x2 bias4[TN][4];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      bias4[j][rg] = u32x2{0u, 0u};
      if (MODE == 1) {
        const int n = n0 + wn0 + j * 32 + 8 * rg + 4 * (l >> 5);
        bias4[j][rg] = *reinterpret_cast<const u32x2*>(e.bias + (n < N ? n : N - 4));
      }
    }
  int gn = n0 + l * 4;
  const bool col_ok = gn < N;
  gn = col_ok ? gn : N - 4;                    // ragged tiles fetch valid memory and ignore it below
#pragma unroll 1
  for (int h = 0; h < 2; ++h) {
    __syncthreads();   // LDS is free: the operand ring (h = 0) or the other half's rows (h = 1)
    for (int r = wave; r < HALF; r += NW) {
      int gm = m0 + h * HALF + r;
      gm = gm < M ? gm : M - 1;
      const float* src = srcm + (int64_t)gm * lds_src + gn;
      const int m0v = __builtin_amdgcn_readfirstlane((int)(size_t)smem + r * PITCH);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                   :
                   : "v"(src), "s"(m0v)
                   : "memory", "m0");
    }
    RV_WAIT_VMCNT(0);
    __syncthreads();
    if (wm0 == h * HALF) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int ml = i * 32 + (l & 31);
        const int gm = m0 + wm0 + ml;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
          for (int rg = 0; rg < 4; ++rg) {
            const int nl = wn0 + j * 32 + 8 * rg + 4 * (l >> 5);
            f32x4* p = reinterpret_cast<f32x4*>(smem + ml * PITCH + nl * 4);
            const f32x4 w = *p;
            f32x4 a = {acc[i][j][4 * rg], acc[i][j][4 * rg + 1], acc[i][j][4 * rg + 2], acc[i][j][4 * rg + 3]};
            f32x4 r;
            if (MODE == 0) {
              r.x = __fmaf_rn(-e.eta, a.x, w.x); r.y = __fmaf_rn(-e.eta, a.y, w.y);
              r.z = __fmaf_rn(-e.eta, a.z, w.z); r.w = __fmaf_rn(-e.eta, a.w, w.w);
              if (e.out && gm < M && n0 + nl < N)
                *reinterpret_cast<f32x4*>((float*)e.out + (int64_t)gm * e.ldo + n0 + nl) = a;
            } else {
              add_bias4(a, bias4[j][rg]);
              r = a + w;
            }
            *p = r;
          }
        }
      }
    }
    __syncthreads();   // the half's results are in LDS
#pragma unroll 1
    for (int rb = 0; rb < RPW; rb += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(smem + (wave + (rb + u) * NW) * PITCH + l * 16);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int gm = m0 + h * HALF + wave + (rb + u) * NW;
        if (gm < M && col_ok) {
          const int64_t o = (int64_t)gm * e.ldo + gn;
          *reinterpret_cast<f32x4*>(dst32 + o) = v[u];
          if (BF16OUT) {
            u32x2 q; q.x = rv_pack_bf16x2(v[u].x, v[u].y); q.y = rv_pack_bf16x2(v[u].z, v[u].w);
            *reinterpret_cast<u32x2*>((uint16_t*)e.out2 + o) = q;
          }
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int NS, int NW, bool AKM, bool BKM, int EPI>
__device__ __forceinline__ void gemm_dtl_body(const uint16_t* __restrict__ A, int64_t lda,
                                              const uint16_t* __restrict__ B, int64_t ldb, int M, int N,
                                              int K, int bm, int bn, const Epi& e) {
  // NW waves laid out 2 (m) x NW/2 (n)
  constexpr int WM = BM / 2, WN = BN / (NW / 2), TM = WM / 32, TN = WN / 32, KSTEPS = BK / 16;
  constexpr int A_BYTES = dtl_tile_bytes(BM, BK), B_BYTES = dtl_tile_bytes(BN, BK);
  constexpr int BUF = A_BYTES + B_BYTES;
  // The eight-wave 256x256 tile runs the pipelined ring below; the four-wave tiles keep the
  // plain ring (loads of tile t+NS-1 right after the barrier that opens tile t).
  constexpr bool PIPELINED = NW == 8 && BM == 256 && BN == 256;
  constexpr int NL = NW;                                                    // loader waves per tile
  constexpr int LPT = Dtl<AKM, BM, BK, NL>::N + Dtl<BKM, BN, BK, NL>::N;   // loads per lane per tile
  static_assert(LPT * (NS - 2) < 64, "vmcnt range");
  char* smem = dtl_smem;

  const int m0 = bm * BM, n0 = bn * BN;
  const int wave = threadIdx.x >> 6;
  const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lw = wave;                 // this wave's share of a tile's loads
  Dtl<AKM, BM, BK, NL> da;
  Dtl<BKM, BN, BK, NL> db;
  dtl_init<AKM, BM, BK, NL>(da, lda, m0, M, lw);
  dtl_init<BKM, BN, BK, NL>(db, ldb, n0, N, lw);
  const int nk = K / BK;
  if constexpr (PIPELINED) {
    // Ring of NS slots, the slot hand-over INSIDE a k-tile.  Before the last k-step of tile s
    // (its fragments are already in registers) the workgroup meets once: tile s+1 has landed
    // and nobody reads tile s's slot any more.  Behind that barrier the first fragments of tile
    // s+1 are read and the loads of tile s+NS go into the slot just left, one behind every
    // few MFMAs of the last k-step - so NS-1 tiles are in flight while one is being used, and
    // the matrix core does not wait at a tile boundary.
    constexpr int NA = Dtl<AKM, BM, BK, NL>::N, NB = Dtl<BKM, BN, BK, NL>::N, LPS = NA + NB;
    constexpr int STRIDE = (TM * TN) / LPS;            // MFMAs per load in the last k-step
    static_assert(STRIDE >= 1 && STRIDE * LPS == TM * TN, "loads are dealt out evenly behind the MFMAs of the last k-step");
    static_assert((NS - 1) * LPS < 64, "vmcnt range");
    unsigned oa[NA], ob[NB];               // per-lane byte offsets of this wave's loads inside a tile
#pragma unroll
    for (int i = 0; i < NA; ++i) oa[i] = (unsigned)da.off[i] * 2u;
#pragma unroll
    for (int i = 0; i < NB; ++i) ob[i] = (unsigned)db.off[i] * 2u;
    auto baseA = [&](int t) { return AKM ? A + (int64_t)t * BK * lda : A + (int64_t)t * BK; };
    auto baseB = [&](int t) { return BKM ? B + (int64_t)t * BK * ldb : B + (int64_t)t * BK; };
    // wait until at most `tiles` of this wave's newest tile loads are still in flight
    auto wait_tiles = [&](int tiles) {
      if (NS >= 5 && tiles >= 4) RV_WAIT_VMCNT(4 * LPS);
      else if (NS >= 5 && tiles == 3) RV_WAIT_VMCNT(3 * LPS);
      else if (NS >= 4 && tiles >= 2) RV_WAIT_VMCNT(2 * LPS);
      else if (NS >= 3 && tiles >= 1) RV_WAIT_VMCNT(1 * LPS);
      else RV_WAIT_VMCNT(0);
    };
    static_assert(NS <= 5, "wait_tiles covers up to four tiles in flight behind the awaited one");
    const int pre = nk < NS ? nk : NS;
    for (int t = 0; t < pre; ++t) {
      const int lb = __builtin_amdgcn_readfirstlane((int)(size_t)(smem + t * BUF) + lw * 1024);
      const uint16_t* pa = baseA(t);
      const uint16_t* pb = baseB(t);
#pragma unroll
      for (int q = 0; q < NA; ++q) dtl_load_s(pa, oa[q], lb + q * NL * 1024);
#pragma unroll
      for (int q = 0; q < NB; ++q) dtl_load_s(pb, ob[q], lb + A_BYTES + q * NL * 1024);
    }
    wait_tiles(pre - 1);
    __syncthreads();
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = dtl_frag<AKM, BM, BK>(smem, wm0 + i * 32, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = dtl_frag<BKM, BN, BK>(smem + A_BYTES, wn0 + j * 32, 0);
    // k-steps 0 .. KSTEPS-2 of the tile in `cur` (fragments of k-step 0 already in fa[0], fb[0])
    auto head_steps = [&](const char* curA, const char* curB) {
#pragma unroll
      for (int kk = 0; kk + 1 < KSTEPS; ++kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[(kk + 1) & 1][i] = dtl_frag<AKM, BM, BK>(curA, wm0 + i * 32, kk + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[(kk + 1) & 1][j] = dtl_frag<BKM, BN, BK>(curB, wn0 + j * 32, kk + 1);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
        constexpr int NREAD = (AKM ? 2 : 1) * TM + (BKM ? 2 : 1) * TN;
        constexpr int NMFMA = TM * TN;
        constexpr int PER = NMFMA / NREAD > 0 ? NMFMA / NREAD : 1;
#pragma unroll
        for (int g = 0; g < NREAD; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
        }
      }
    };
    auto next_frags = [&](const char* nxtA) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[0][i] = dtl_frag<AKM, BM, BK>(nxtA, wm0 + i * 32, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[0][j] = dtl_frag<BKM, BN, BK>(nxtA + A_BYTES, wn0 + j * 32, 0);
    };
    static_assert((KSTEPS & 1) == 0, "the next tile's first fragments go to buffer 0");
    constexpr int L = (KSTEPS - 1) & 1;      // the last k-step's fragments are in fa[L], fb[L]
    int slot = 0;                            // ring slot of tile s
    int s = 0;
    for (; s + NS < nk; ++s) {               // passes that still have a tile s+NS to fetch
      const char* curA = smem + slot * BUF;
      const int nslot = slot + 1 == NS ? 0 : slot + 1;
      head_steps(curA, curA + A_BYTES);
      RV_WAIT_VMCNT((NS - 2) * LPS);         // tile s+1 (tiles s+2 .. s+NS-1 may still fly)
      __syncthreads();                       // all of tile s+1 is in LDS; all fragment reads of tile s are done
      next_frags(smem + nslot * BUF);
      const int lb = __builtin_amdgcn_readfirstlane((int)(size_t)(smem + slot * BUF) + lw * 1024);
      const uint16_t* pa = baseA(s + NS);
      const uint16_t* pb = baseB(s + NS);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int m = i * TN + j;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[L][j], fa[L][i], acc[i][j], 0, 0, 0);
          if (m % STRIDE == 0) {
            const int q = m / STRIDE;
            __builtin_amdgcn_sched_barrier(0);
            if (q < NA) dtl_load_s(pa, oa[q], lb + q * NL * 1024);
            else dtl_load_s(pb, ob[q - NA], lb + A_BYTES + (q - NA) * NL * 1024);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      slot = nslot;
    }
    for (; s + 1 < nk; ++s) {                // the last NS-1 hand-overs: nothing left to fetch
      const char* curA = smem + slot * BUF;
      const int nslot = slot + 1 == NS ? 0 : slot + 1;
      head_steps(curA, curA + A_BYTES);
      wait_tiles(nk - 2 - s);                // tiles s+2 .. nk-1 may still fly
      __syncthreads();
      next_frags(smem + nslot * BUF);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[L][j], fa[L][i], acc[i][j], 0, 0, 0);
      slot = nslot;
    }
    {
      const char* curA = smem + slot * BUF;
      head_steps(curA, curA + A_BYTES);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[L][j], fa[L][i], acc[i][j], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
      if (t < nk) {
        dtl_issue<AKM, BM, BK, NL>(da, A, lda, t * BK, smem + t * BUF, lw);
        dtl_issue<BKM, BN, BK, NL>(db, B, ldb, t * BK, smem + t * BUF + A_BYTES, lw);
      }
    int stage = 0;               // ring slot of tile `it`
    int fill = NS - 1;           // ring slot the next issued tile goes to
    for (int it = 0; it < nk; ++it) {
      // tile `it` has landed once at most the loads of the newer tiles are outstanding
      const int newer = nk - 1 - it;
      if (NS >= 4 && newer >= NS - 2) RV_WAIT_VMCNT(LPT * (NS - 2));
      else if (NS >= 3 && newer >= 1) { if (NS >= 4 && newer >= 2) RV_WAIT_VMCNT(LPT * 2); else RV_WAIT_VMCNT(LPT * 1); }
      else RV_WAIT_VMCNT(0);
      __syncthreads();           // everyone's part of tile `it` is in LDS; everyone left tile it-1
      if (it + NS - 1 < nk) {
        dtl_issue<AKM, BM, BK, NL>(da, A, lda, (it + NS - 1) * BK, smem + fill * BUF, lw);
        dtl_issue<BKM, BN, BK, NL>(db, B, ldb, (it + NS - 1) * BK, smem + fill * BUF + A_BYTES, lw);
      }
      const char* curA = smem + stage * BUF;
      const char* curB = curA + A_BYTES;
      bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[0][i] = dtl_frag<AKM, BM, BK>(curA, wm0 + i * 32, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[0][j] = dtl_frag<BKM, BN, BK>(curB, wn0 + j * 32, 0);
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        if (kk + 1 < KSTEPS) {
#pragma unroll
          for (int i = 0; i < TM; ++i) fa[(kk + 1) & 1][i] = dtl_frag<AKM, BM, BK>(curA, wm0 + i * 32, kk + 1);
#pragma unroll
          for (int j = 0; j < TN; ++j) fb[(kk + 1) & 1][j] = dtl_frag<BKM, BN, BK>(curB, wn0 + j * 32, kk + 1);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
        if (kk + 1 < KSTEPS) {
          constexpr int NREAD = (AKM ? 2 : 1) * TM + (BKM ? 2 : 1) * TN;
          constexpr int NMFMA = TM * TN;
          constexpr int PER = NMFMA / NREAD > 0 ? NMFMA / NREAD : 1;
#pragma unroll
          for (int g = 0; g < NREAD; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
          }
        }
      }
      stage = stage + 1 == NS ? 0 : stage + 1;
      fill = fill + 1 == NS ? 0 : fill + 1;
    }
  }
  if constexpr (staged_epi(EPI)) {
    write_tile_staged<BM, BN, 64 * NW, TM, TN, EPI>(acc, e, m0, n0, wm0, wn0, M, N, smem);
  } else if constexpr (EPI == EPI_F32_UPD) {
    if (e.upd_w) f32_tile_through_lds<BM, BN, NW, TM, TN, 0, true>(acc, e, m0, n0, wm0, wn0, M, N, smem);   // workgroup-uniform
    else write_tile<TM, TN, EPI>(acc, e, m0 + wm0, n0 + wn0, M, N);
  } else if constexpr (epi_has_resid(EPI) && PIPELINED && RV_RESID_LDS) {
    f32_tile_through_lds<BM, BN, NW, TM, TN, 1, EPI == EPI_F32_BIAS_RESID_BF16>(acc, e, m0, n0, wm0, wn0, M, N, smem);
  } else {
    write_tile<TM, TN, EPI>(acc, e, m0 + wm0, n0 + wn0, M, N);
  }
}

template <int BM, int BN, int BK, int NS, int NW, int WPE, bool AKM, bool BKM, int EPI>
__global__ __launch_bounds__(64 * NW, WPE) void gemm_dtl_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                 const uint16_t* __restrict__ B, int64_t ldb,
                                                                 int M, int N, int K, int tiles_m, int tiles_n,
                                                                 int band_rows, Epi e) {
  int bm, bn;
  tile_of_block(tiles_m, tiles_n, band_rows, bm, bn);
  gemm_dtl_body<BM, BN, BK, NS, NW, AKM, BKM, EPI>(A, lda, B, ldb, M, N, K, bm, bn, e);
}

// Several independent products of one kind in a single launch (the four weight-gradient
// products of a decoder block): a workgroup finds its problem from the running tile count.
// One launch fills the chip where four small grids would each leave most CUs idle.
struct GroupedProblem {
  const uint16_t* A; const uint16_t* B; float* out;
  float* upd_w; uint16_t* upd_ver; float eta;
  int lda, ldb, ldo, M, N, K, tiles_m, tiles_n, first_tile;
};
struct GroupedArgs {
  GroupedProblem p[RV_GEMM_GROUP_MAX];
  int count;
};

template <int BM, int BN, int BK, int NS, int NW, int WPE>
__global__ __launch_bounds__(64 * NW, WPE) void gemm_dtl_grouped_wgrad_kernel(GroupedArgs ga) {
  // Workgroup ids are dealt to the 8 XCDs in turn, and each XCD pulls its operand panels
  // through its own L2.  Give XCD g a CONTIGUOUS range of the tile numbering (so it works on
  // one problem at a time, not on a slice of all of them) and number a problem's tiles in bands
  // of two tile rows, column by column (so a run of 8 tiles is a 2 x 4 patch: 6 operand panels).
  const int total = gridDim.x, base = total / 8, rem = total % 8;
  const int g = blockIdx.x % 8, i = blockIdx.x / 8;
  const int v = g * base + (g < rem ? g : rem) + i;
  int pi = 0;
#pragma unroll
  for (int k = 1; k < RV_GEMM_GROUP_MAX; ++k)
    if (k < ga.count && v >= ga.p[k].first_tile) pi = k;
  const GroupedProblem& q = ga.p[pi];
  const int local = v - q.first_tile;
  constexpr int GB = 2;
  const int band = local / (GB * q.tiles_n), first_row = band * GB;
  const int rows = q.tiles_m - first_row < GB ? q.tiles_m - first_row : GB;
  const int in = local - band * GB * q.tiles_n;
  Epi e{q.out, q.ldo, q.upd_ver, nullptr, nullptr, 0, nullptr, q.upd_w, q.eta, nullptr};
  gemm_dtl_body<BM, BN, BK, NS, NW, true, true, EPI_F32_UPD>(q.A, q.lda, q.B, q.ldb, q.M, q.N, q.K, first_row + in % rows,
                                                      in / rows, e);
}

template <int BM, int BN, int BK, int NS, int NW, int WPE, bool AKM, bool BKM, int EPI>
rv_status launch_dtl(const rv_gemm_args& g, hipStream_t st) {
  constexpr int ring = NS * (dtl_tile_bytes(BM, BK) + dtl_tile_bytes(BN, BK));
  // the GELU' epilogue keeps two rows of fp32 column sums (one per wave row) behind the image
  constexpr int image = staged_epi(EPI) ? BM * stage_pitch(BN) + (EPI == EPI_BF16_DGELU ? 2 * BN * 4 : 0)
                        : (epi_has_resid(EPI) && NW == 8 && BM == 256 && BN == 256 ? upd_image_bytes(BM, BN) : 0);
  constexpr int smem = ring > image ? ring : image;
  auto kern = gemm_dtl_kernel<BM, BN, BK, NS, NW, WPE, AKM, BKM, EPI>;
  // once per instantiation; a function-local static is initialised exactly once, also under threads
  static const hipError_t configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (configured != hipSuccess) return RV_E_DEVICE;
  int tm = (g.M + BM - 1) / BM, tn = (g.N + BN - 1) / BN;
  Epi e{g.out, g.ldo, g.out2, g.bias, g.resid, g.ldr, g.zin, nullptr, 0.f, g.epi == EPI_BF16_DGELU ? g.colpart : nullptr};
  g.colpart_rows = (g.M + BM - 1) / BM;
  const int ntiles = tm * tn;
  // Measured: alone, the XCD-banded map pays only for the small tile.  Inside a stage step a
  // launch holds about a third of every XCD's CUs, and what an XCD runs of it at one time should
  // share operand panels: bands of 8 tile rows (2 for 32 or more tile rows, either tile size)
  // against the natural order: stage steps -1.3 % / -0.6 % / -1.9 % (configs 5 / 3 / 2).
  int band = 8;
  if (g.sharing != 0) band = tm >= 32 ? 2 : 8;
  else if (!(BM == 128 && BN == 128)) tm = -tm;
  hipLaunchKernelGGL(kern, dim3(ntiles), dim3(64 * NW), smem, st, g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K,
                     tm, tn, band, e);
  return rv_launch_status();
}

// Tile choice (codes: 5256, 2256, 2192, 2128).
//   5256  256x256, eight waves of 128x64, BK 32, ring of four slots run in the pipelined form
//         (three tiles in flight, loads dealt out behind the MFMAs), one workgroup per CU:
//         lowest LDS traffic per MFMA, two waves per SIMD cover each other's stalls;
//   2192  128x256, four waves of 64x128, BK 32, three stages, two workgroups per CU;
//   2128  128x128, four waves of 64x64, BK 64, two stages, two workgroups per CU: fills the
//         chip on small outputs.
// The automatic choice minimises  rounds * tile_area * workgroups_per_CU / efficiency  with
// rounds = ceil(tiles / (256 CUs * workgroups_per_CU)); efficiencies are measured ratios.
template <bool AKM, bool BKM, int EPI>
rv_status pick_tile(const rv_gemm_args& g, hipStream_t st) {
  auto cost = [&](int bm, int bn, int bpc, double eff) {
    const long tiles = (long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn);
    const long rounds = (tiles + 256 * bpc - 1) / (256 * bpc);
    return (double)rounds * bm * bn * bpc / eff;
  };
  int tile = g.tile;
  if (tile == 0 && g.sharing) {
    // Measured inside the stage step (configs 2, 3, 5): what a launch leaves of the chip is
    // used by the other streams, so CU time per flop counts for more than its own duration.
    const long t256 = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (g.sharing == 2 || t256 >= 128) tile = 5256;
  }
  if (tile == 0) {
    const double c256 = cost(256, 256, 1, 1.0), c192 = cost(128, 256, 2, 0.92), c128 = cost(128, 128, 2, 0.85);
    tile = c256 <= c192 && c256 <= c128 ? 5256 : (c192 <= c128 ? 2192 : 2128);
  }
  if (tile == 2256) return launch_dtl<256, 256, 32, 4, 4, 1, AKM, BKM, EPI>(g, st);
  if (tile == 2192) return launch_dtl<128, 256, 32, 3, 4, 2, AKM, BKM, EPI>(g, st);
  if (tile == 2128) return launch_dtl<128, 128, 64, 2, 4, 2, AKM, BKM, EPI>(g, st);
  if (tile == 5256) return launch_dtl<256, 256, 32, 4, 8, 2, AKM, BKM, EPI>(g, st);
  return RV_E_INVAL;
}

}  // namespace

rv_status rv_gemm_bf16(const rv_gemm_args& g, hipStream_t st) {
  if (!g.A || !g.B || !g.out || g.M < 8 || g.N < 8 || g.K < 64) return RV_E_INVAL;
  if (g.K % 64 || g.N % 8 || g.M % 8 || g.lda % 8 || g.ldb % 8 || g.ldo % 4) return RV_E_INVAL;
  if ((((uintptr_t)g.A) | ((uintptr_t)g.B) | ((uintptr_t)g.out)) & 15) return RV_E_INVAL;
  // bf16 outputs (and the pre-activation input of GELU') move in 16-byte row pieces: pitch % 8
  if ((staged_epi(g.epi) || g.epi == EPI_F32_BIAS_RESID_BF16) && g.ldo % 8) return RV_E_INVAL;
  if (staged_epi(g.epi) && g.epi == EPI_BF16_BIAS_GELU && (((uintptr_t)g.out2) & 15)) return RV_E_INVAL;
  if (g.epi == EPI_BF16_DGELU && (((uintptr_t)g.zin) & 15)) return RV_E_INVAL;
  // tile offsets are kept in 32 bits
  if ((int64_t)(g.a_kmajor ? g.K : g.M) * g.lda >= (1ll << 31) || (int64_t)(g.b_kmajor ? g.K : g.N) * g.ldb >= (1ll << 31))
    return RV_E_INVAL;
  const bool need_bias = g.epi == EPI_BF16_BIAS || g.epi == EPI_F32_BIAS_RESID ||
                         g.epi == EPI_BF16_BIAS_GELU || g.epi == EPI_F32_BIAS_RESID_BF16;
  if (need_bias && (!g.bias || (((uintptr_t)g.bias) & 7))) return RV_E_INVAL;
  if ((g.epi == EPI_F32_BIAS_RESID || g.epi == EPI_F32_BIAS_RESID_BF16) &&
      (!g.resid || g.ldr % 4 || (((uintptr_t)g.resid) & 15)))
    return RV_E_INVAL;
  if ((g.epi == EPI_BF16_BIAS_GELU || g.epi == EPI_F32_BIAS_RESID_BF16) && !g.out2) return RV_E_INVAL;
  if (g.epi == EPI_BF16_DGELU && !g.zin) return RV_E_INVAL;
  // only the layout/epilogue pairs the stage uses are instantiated
  if (!g.a_kmajor && g.b_kmajor) {          // forward products
    switch (g.epi) {
      case EPI_BF16_BIAS: return pick_tile<false, true, EPI_BF16_BIAS>(g, st);
      case EPI_F32_BIAS_RESID: return pick_tile<false, true, EPI_F32_BIAS_RESID>(g, st);
      case EPI_F32_BIAS_RESID_BF16: return pick_tile<false, true, EPI_F32_BIAS_RESID_BF16>(g, st);
      case EPI_BF16_BIAS_GELU: return pick_tile<false, true, EPI_BF16_BIAS_GELU>(g, st);
    }
  } else if (!g.a_kmajor && !g.b_kmajor) {  // input-gradient products
    switch (g.epi) {
      case EPI_BF16: return pick_tile<false, false, EPI_BF16>(g, st);
      case EPI_BF16_DGELU: return pick_tile<false, false, EPI_BF16_DGELU>(g, st);
    }
  } else if (g.a_kmajor && g.b_kmajor) {    // weight-gradient products
    if (g.epi == EPI_F32) return pick_tile<true, true, EPI_F32>(g, st);
  }
  return RV_E_INVAL;
}

namespace {
template <int BM, int BN, int BK, int NS, int NW>
rv_status launch_grouped(const rv_gemm_args* gs, int count, hipStream_t st) {
  GroupedArgs ga;
  int tiles = 0;
  for (int k = 0; k < count; ++k) {
    const rv_gemm_args& g = gs[k];
    GroupedProblem& q = ga.p[k];
    q.A = g.A; q.B = g.B; q.out = g.store_out ? (float*)g.out : nullptr;
    q.upd_w = g.upd_w; q.upd_ver = g.upd_ver; q.eta = g.upd_eta;
    q.lda = (int)g.lda; q.ldb = (int)g.ldb; q.ldo = (int)g.ldo; q.M = g.M; q.N = g.N; q.K = g.K;
    q.tiles_m = (g.M + BM - 1) / BM;
    q.tiles_n = (g.N + BN - 1) / BN;
    q.first_tile = tiles;
    tiles += q.tiles_m * q.tiles_n;
  }
  for (int k = count; k < RV_GEMM_GROUP_MAX; ++k) ga.p[k] = ga.p[0];
  ga.count = count;
  constexpr int ring = NS * (dtl_tile_bytes(BM, BK) + dtl_tile_bytes(BN, BK));
  constexpr int smem = ring > upd_image_bytes(BM, BN) ? ring : upd_image_bytes(BM, BN);
  static_assert(smem <= 160 * 1024, "LDS of one CU");
  auto kern = gemm_dtl_grouped_wgrad_kernel<BM, BN, BK, NS, NW, 2>;
  static const hipError_t configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (configured != hipSuccess) return RV_E_DEVICE;
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(64 * NW), smem, st, ga);
  return rv_launch_status();
}
}  // namespace

rv_status rv_gemm_wgrad_grouped(const rv_gemm_args* gs, int count, hipStream_t st) {
  if (!gs || count < 1 || count > RV_GEMM_GROUP_MAX) return RV_E_INVAL;
  for (int k = 0; k < count; ++k) {
    const rv_gemm_args& g = gs[k];
    if (!g.A || !g.B || !g.out || !g.a_kmajor || !g.b_kmajor || g.epi != EPI_F32) return RV_E_INVAL;
    if (g.M < 8 || g.N < 8 || g.K < 64 || g.K % 64 || g.N % 8 || g.M % 8 || g.lda % 8 || g.ldb % 8 || g.ldo % 4)
      return RV_E_INVAL;
    if ((((uintptr_t)g.A) | ((uintptr_t)g.B) | ((uintptr_t)g.out)) & 15) return RV_E_INVAL;
    if ((int64_t)g.K * g.lda >= (1ll << 31) || (int64_t)g.K * g.ldb >= (1ll << 31)) return RV_E_INVAL;
    if ((g.upd_w != nullptr) != (g.upd_ver != nullptr)) return RV_E_INVAL;
    if (!g.upd_w && !g.store_out) return RV_E_INVAL;
    if ((((uintptr_t)g.upd_w) & 15) || (((uintptr_t)g.upd_ver) & 7)) return RV_E_INVAL;
  }
  // 256x256 tiles, eight waves (measured against 128x128 and 128x256 tiles, alone and inside the
  // stage step of configs 2, 3 and 5: fewest LDS bytes per MFMA, so it takes the least CU time
  // from the kernels that run beside it, and the step is 3-4 % shorter)
  return launch_grouped<256, 256, 32, 4, 8>(gs, count, st);
}

extern "C" rv_status rv_k_gemm_bf16(const void* A, int64_t lda, int a_kmajor, const void* B, int64_t ldb,
                                    int b_kmajor, int M, int N, int K, int epilogue, void* out, int64_t ldo,
                                    void* out2, const void* bias, const float* resid, int64_t ldr,
                                    const void* zin, int tile, void* stream) {
  rv_gemm_args g;
  g.A = (const uint16_t*)A; g.lda = lda; g.a_kmajor = a_kmajor;
  g.B = (const uint16_t*)B; g.ldb = ldb; g.b_kmajor = b_kmajor;
  g.M = M; g.N = N; g.K = K; g.epi = epilogue; g.out = out; g.ldo = ldo; g.out2 = out2;
  g.bias = (const uint16_t*)bias; g.resid = resid; g.ldr = ldr; g.zin = (const uint16_t*)zin; g.tile = tile;
  return rv_gemm_bf16(g, (hipStream_t)stream);
}

extern "C" rv_status rv_k_gemm_wgrad_grouped(int count, const void* const* X, const int64_t* lda,
                                             const void* const* dY, const int64_t* ldb, const int* M, const int* N,
                                             int K, float* const* dW, void* stream) {
  if (count < 1 || count > RV_GEMM_GROUP_MAX || !X || !lda || !dY || !ldb || !M || !N || !dW) return RV_E_INVAL;
  rv_gemm_args g[RV_GEMM_GROUP_MAX];
  for (int k = 0; k < count; ++k) {
    g[k].A = (const uint16_t*)X[k]; g[k].lda = lda[k]; g[k].a_kmajor = 1;
    g[k].B = (const uint16_t*)dY[k]; g[k].ldb = ldb[k]; g[k].b_kmajor = 1;
    g[k].M = M[k]; g[k].N = N[k]; g[k].K = K; g[k].epi = EPI_F32; g[k].out = dW[k]; g[k].ldo = N[k];
  }
  return rv_gemm_wgrad_grouped(g, count, (hipStream_t)stream);
}
