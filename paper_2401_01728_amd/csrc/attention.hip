// Causal self-attention of the decoder block, forward and backward, on bf16 MFMA with
// fp32 softmax statistics (a piece of a peer's forward_pass and of its exact gradient,
// paper Alg. 1 / Eq. 2).  q|k|v live in one [tokens, 3*d_model] matrix (column thirds,
// heads contiguous inside a third); heads are merged in the [tokens, d_model] output.
//
// All three kernels keep the score tile in registers and never write it to memory.
// A wave owns 32 rows of one operand (queries, or keys in the dK/dV kernel), held as MFMA
// B-fragments for the whole kernel; the other side streams through LDS in tiles of 64
// rows shared by the four waves of a workgroup.
//
// Scores are computed TRANSPOSED relative to the side a wave owns, so that the owned
// index is the lane (lane % 32) and the streamed index runs over a lane's 16 accumulator
// registers.  Row statistics (max, sum, lse, D) are then per-lane scalars, and the
// probability tile is already in the register layout of an MFMA B operand for the second
// product (contraction over the streamed index) - no shuffles, no LDS round trip.  The A
// operand of that product is the streamed tile transposed, which the LDS transpose read
// (ds_read_b64_tr_b16) delivers with a row order matching the accumulator layout.
//
// Softmax runs in base 2: s2 = s * (log2(e)/sqrt(dh)), p = exp2(s2 - m).  The forward
// stores lse2 = m + log2(sum); the backward recomputes p = exp2(s2 - lse2).
// Backward is split in two deterministic kernels (no atomics): one accumulates dQ per query
// tile (and leaves D = rowsum(dO * O) behind), one accumulates dK and dV per key tile over the
// queries that see it.
#include <mutex>
#include "internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int TILE = 64;    // streamed rows per LDS tile
constexpr int WROWS = 32;   // rows a wave owns
constexpr int BROWS = 128;  // rows a workgroup owns

template <int DH> struct L {
  static constexpr int PKC = DH * 2 + 16;          // k-contiguous pitch (bytes)
  static constexpr int PKM = DH * 2 + 64;          // transpose-read pitch (bytes)
  static constexpr int KC_BYTES = TILE * PKC;
  static constexpr int KM_BYTES = TILE * PKM;
  static constexpr int CHUNKS = TILE * DH / 8 / kThreads;  // 16-byte chunks per lane per tile
};

// global [TILE rows][DH] (row pitch ld elements) -> registers
template <int DH>
__device__ __forceinline__ void g2r(u32x4* v, const uint16_t* __restrict__ g, int64_t ld) {
#pragma unroll
  for (int i = 0; i < L<DH>::CHUNKS; ++i) {
    const int idx = threadIdx.x + kThreads * i;
    const int row = idx / (DH / 8), c = idx % (DH / 8);
    v[i] = *reinterpret_cast<const u32x4*>(g + (int64_t)row * ld + c * 8);
  }
}
template <int DH, int PITCH>
__device__ __forceinline__ void r2s(const u32x4* v, char* lds) {
#pragma unroll
  for (int i = 0; i < L<DH>::CHUNKS; ++i) {
    const int idx = threadIdx.x + kThreads * i;
    const int row = idx / (DH / 8), c = idx % (DH / 8);
    *reinterpret_cast<u32x4*>(lds + row * PITCH + c * 16) = v[i];
  }
}

// A fragment, rows row0 + lane%32, k = dh index 16*kk + 8*(lane/32) .. +7, from a k-contiguous tile
template <int DH>
__device__ __forceinline__ bf16x8 frag_kc(const char* lds, int row0, int kk) {
  const int l = threadIdx.x & 63;
  return *reinterpret_cast<const bf16x8*>(lds + (row0 + (l & 31)) * L<DH>::PKC + kk * 32 + (l >> 5) * 16);
}

// A fragment of the TRANSPOSED tile: m = dh index col0 + lane%32, k-slots e = 0..7 of lane
// group g = lane/32 hold tile rows  row0 + 4g + e  (e < 4)  and  row0 + 8 + 4g + (e-4):
// exactly the rows a lane's accumulator registers 8*ks .. 8*ks+7 correspond to.
template <int DH>
__device__ __forceinline__ bf16x8 frag_tr(const char* lds, int row0, int col0) {
  const int l = threadIdx.x & 63;
  const int q = l >> 4, i = l & 15;
  const int row = row0 + 4 * (q >> 1) + (i >> 2);
  const int col = col0 + 16 * (q & 1) + 4 * (i & 3);
  const char* p = lds + row * L<DH>::PKM + col * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p + 8 * L<DH>::PKM));
  s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

// registers 8*ks .. 8*ks+7 of an accumulator tile -> bf16 B fragment
__device__ __forceinline__ bf16x8 pack_frag(const f32x16& a, int ks) {
  u32x4 r;
  r.x = rv_pack_bf16x2(a[8 * ks + 0], a[8 * ks + 1]);
  r.y = rv_pack_bf16x2(a[8 * ks + 2], a[8 * ks + 3]);
  r.z = rv_pack_bf16x2(a[8 * ks + 4], a[8 * ks + 5]);
  r.w = rv_pack_bf16x2(a[8 * ks + 6], a[8 * ks + 7]);
  return __builtin_bit_cast(bf16x8, r);
}

// streamed-row index (within a 32-row sub tile) of accumulator register r for lane group g
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// owned-side fragments straight from global: rows tok0 + lane%32, all of DH
template <int DH>
__device__ __forceinline__ void load_owned(bf16x8* f, const uint16_t* __restrict__ g, int64_t ld) {
  const int l = threadIdx.x & 63;
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk)
    f[kk] = *reinterpret_cast<const bf16x8*>(g + (int64_t)(l & 31) * ld + kk * 16 + (l >> 5) * 8);
}

// write a transposed accumulator (lane = row, registers = 4-column groups) as bf16
template <int DH>
__device__ __forceinline__ void store_owned(const f32x16* acc, float mul, uint16_t* __restrict__ g, int64_t ld) {
  const int l = threadIdx.x & 63, grp = l >> 5;
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      u32x2 o;
      o.x = rv_pack_bf16x2(acc[dt][4 * rg] * mul, acc[dt][4 * rg + 1] * mul);
      o.y = rv_pack_bf16x2(acc[dt][4 * rg + 2] * mul, acc[dt][4 * rg + 3] * mul);
      *reinterpret_cast<u32x2*>(g + (int64_t)(l & 31) * ld + dt * 32 + 8 * rg + 4 * grp) = o;
    }
}

// Column sums of the same accumulator over the wave's 32 rows (the lanes of a half wave), into
// dst[0 .. DH): one partial row of the bias gradient that belongs to this slice of dqkv.  The
// sums run over the fp32 values in a fixed butterfly order (rv_half_wave_sum).
template <int DH>
__device__ __forceinline__ void colsum_owned(const f32x16* acc, float mul, float* __restrict__ dst) {
  const int l = threadIdx.x & 63, grp = l >> 5;
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      f32x4 v;
      v.x = rv_half_wave_sum(acc[dt][4 * rg] * mul); v.y = rv_half_wave_sum(acc[dt][4 * rg + 1] * mul);
      v.z = rv_half_wave_sum(acc[dt][4 * rg + 2] * mul); v.w = rv_half_wave_sum(acc[dt][4 * rg + 3] * mul);
      if ((l & 31) == 0) *reinterpret_cast<f32x4*>(dst + dt * 32 + 8 * rg + 4 * grp) = v;
    }
}

// Workgroup -> (row block, head, sequence).  Causal work per row block is a ramp, and
// consecutive workgroup ids go to the 8 XCDs in turn: the block index must be the SLOWEST
// digit of the id, or whole XCDs get only long (or only short) blocks and the kernel lasts as
// long as the unluckiest XCD (measured: 1.2x - 1.7x).  rank 0 is the heaviest block, so the
// long blocks also start first.
__device__ __forceinline__ void attn_block(int H, int nseq, int& rank, int& h, int& b) {
  const int per = H * nseq;
  rank = blockIdx.x / per;
  const int rest = blockIdx.x % per;
  h = rest % H; b = rest / H;
}

// ----------------------------------------------------------------------------------------
// forward
// ----------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(const uint16_t* __restrict__ qkv, int64_t ld,
                                                            uint16_t* __restrict__ out, int64_t ldo,
                                                            float* __restrict__ lse2, int S, int d, int H,
                                                            int nseq, float c2) {
  extern __shared__ __align__(16) char smem[];
  constexpr int BUF = L<DH>::KC_BYTES + L<DH>::KM_BYTES;   // K tile (k-contiguous) + V tile (transpose-read)
  const int nblk = (S + BROWS - 1) / BROWS;
  int rank, h, b;
  attn_block(H, nseq, rank, h, b);
  const int qb = nblk - 1 - rank;                          // long rows first
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, grp = l >> 5;
  const int q0 = qb * BROWS + wave * WROWS;
  const bool active = q0 < S;
  const int64_t tok0 = (int64_t)b * S;
  const uint16_t* Kg = qkv + tok0 * ld + d + h * DH;
  const uint16_t* Vg = qkv + tok0 * ld + 2 * d + h * DH;

  bf16x8 qf[DH / 16];
  if (active) load_owned<DH>(qf, qkv + (tok0 + q0) * ld + h * DH, ld);
  f32x16 o[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;
  const int qi = q0 + (l & 31);

  const int nkt = min(S, (qb + 1) * BROWS) / TILE;
  u32x4 kr[L<DH>::CHUNKS], vr[L<DH>::CHUNKS];
  g2r<DH>(kr, Kg, ld); g2r<DH>(vr, Vg, ld);
  r2s<DH, L<DH>::PKC>(kr, smem); r2s<DH, L<DH>::PKM>(vr, smem + L<DH>::KC_BYTES);
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const char* Ks = smem + (kt & 1) * BUF;
    const char* Vs = Ks + L<DH>::KC_BYTES;
    if (kt + 1 < nkt) {
      g2r<DH>(kr, Kg + (int64_t)(kt + 1) * TILE * ld, ld);
      g2r<DH>(vr, Vg + (int64_t)(kt + 1) * TILE * ld, ld);
    }
    const int k0 = kt * TILE;
    if (active && k0 <= q0 + WROWS - 1) {
      f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
      for (int kk = 0; kk < DH / 16; ++kk)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
          s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<DH>(Ks, sub * 32, kk), qf[kk], s[sub], 0, 0, 0);
      // running max m is kept in the scaled base-2 domain; the scale (> 0) commutes with max,
      // so the row max is taken over raw scores and p = exp2(s*c2 - m) is one FMA + one exp
      // only tiles that straddle the diagonal pay for the causal mask (wave-uniform branch)
      const bool diag = k0 + TILE - 1 > q0;
      float mx = -INFINITY;
      if (diag) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = s[sub][r];
            if (k0 + sub * 32 + acc_row(r, grp) > qi) v = -INFINITY;
            s[sub][r] = v;
            mx = fmaxf(mx, v);
          }
      } else {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sub][r]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m, mx * c2);
      const float alpha = __builtin_amdgcn_exp2f(m - mn);
      m = mn;
      float ps = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(__fmaf_rn(s[sub][r], c2, -mn));
          s[sub][r] = p;
          ps += p;
        }
      lsum = lsum * alpha + ps;
      // once the running maxima have settled alpha is exactly 1 in every lane: skip the rescale
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt) o[dt] *= alpha;
      }
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const bf16x8 pf = pack_frag(s[sub], ks);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt)
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(Vs, sub * 32 + ks * 16, dt * 32), pf,
                                                            o[dt], 0, 0, 0);
        }
    }
    if (kt + 1 < nkt) {
      char* nb = smem + ((kt + 1) & 1) * BUF;
      r2s<DH, L<DH>::PKC>(kr, nb); r2s<DH, L<DH>::PKM>(vr, nb + L<DH>::KC_BYTES);
    }
    __syncthreads();
  }
  if (!active) return;
  const float tot = lsum + __shfl_xor(lsum, 32, 64);
  store_owned<DH>(o, 1.0f / tot, out + (tok0 + q0) * ldo + h * DH, ldo);
  if (grp == 0) lse2[((int64_t)b * H + h) * S + qi] = m + __builtin_amdgcn_logf(tot);   // v_log_f32 is log2
}

// ----------------------------------------------------------------------------------------
// backward, part 2 (launched second: it reads the D the dQ kernel stores): dK and dV.
// A wave owns 32 keys (lane = key); queries stream.
// ----------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_bwd_kv_kernel(const uint16_t* __restrict__ qkv, int64_t ld,
                                                               const uint16_t* __restrict__ dout, int64_t ldo,
                                                               const float* __restrict__ lse2,
                                                               const float* __restrict__ Dv,
                                                               uint16_t* __restrict__ dqkv, int S, int d, int H,
                                                               int nseq, float c2, float scale,
                                                               float* __restrict__ colpart) {
  extern __shared__ __align__(16) char smem[];
  char* Qkc = smem;                         // Q tile, k-contiguous (for S = Q K^T)
  char* Qkm = Qkc + L<DH>::KC_BYTES;        // Q tile, transpose-read (for dK^T = Q^T dS)
  char* Okc = Qkm + L<DH>::KM_BYTES;        // dO tile, k-contiguous (for dP = dO V^T)
  char* Okm = Okc + L<DH>::KC_BYTES;        // dO tile, transpose-read (for dV^T = dO^T P)
  float* stat = reinterpret_cast<float*>(Okm + L<DH>::KM_BYTES);   // lse2[64], D[64]

  int jb, h, b;                             // the first key block sees every query: heaviest
  attn_block(H, nseq, jb, h, b);
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, grp = l >> 5;
  const int j0 = jb * BROWS + wave * WROWS;
  const bool active = j0 < S;
  const int64_t tok0 = (int64_t)b * S;
  const uint16_t* Qg = qkv + tok0 * ld + h * DH;
  const uint16_t* Og = dout + tok0 * ldo + h * DH;
  const float* lse_g = lse2 + ((int64_t)b * H + h) * S;
  const float* D_g = Dv + ((int64_t)b * H + h) * S;

  bf16x8 kf[DH / 16], vf[DH / 16];
  if (active) {
    load_owned<DH>(kf, qkv + (tok0 + j0) * ld + d + h * DH, ld);
    load_owned<DH>(vf, qkv + (tok0 + j0) * ld + 2 * d + h * DH, ld);
  }
  f32x16 dk[DH / 32], dv[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) { dk[dt] = zero16(); dv[dt] = zero16(); }
  const int ji = j0 + (l & 31);

  // The next tile's global loads are in flight while the current tile is computed; they are
  // parked in LDS after the barrier that ends the compute phase.
  const int nit = S / TILE;
  const int it0 = jb * (BROWS / TILE);
  u32x4 rq[L<DH>::CHUNKS], ro[L<DH>::CHUNKS];
  float rstat = 0.f;
  auto fetch = [&](int it) {
    const int i0 = it * TILE;
    g2r<DH>(rq, Qg + (int64_t)i0 * ld, ld);
    g2r<DH>(ro, Og + (int64_t)i0 * ldo, ldo);
    if (threadIdx.x < TILE) rstat = lse_g[i0 + threadIdx.x];
    else if (threadIdx.x < 2 * TILE) rstat = D_g[i0 + threadIdx.x - TILE];
  };
  auto park = [&]() {
    r2s<DH, L<DH>::PKC>(rq, Qkc); r2s<DH, L<DH>::PKM>(rq, Qkm);
    r2s<DH, L<DH>::PKC>(ro, Okc); r2s<DH, L<DH>::PKM>(ro, Okm);
    if (threadIdx.x < 2 * TILE) stat[threadIdx.x] = rstat;
  };
  if (it0 < nit) { fetch(it0); park(); }
  __syncthreads();
  for (int it = it0; it < nit; ++it) {
    const int i0 = it * TILE;
    if (it + 1 < nit) fetch(it + 1);
    if (active) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int is = i0 + sub * 32;
        if (is + 31 < j0) continue;                       // every query of this sub tile precedes the keys
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int kk = 0; kk < DH / 16; ++kk) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<DH>(Qkc, sub * 32, kk), kf[kk], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<DH>(Okc, sub * 32, kk), vf[kk], dp, 0, 0, 0);
        }
        const bool diag = is < j0 + WROWS - 1;           // wave-uniform: only diagonal tiles mask
        if (diag) {
#pragma unroll
          for (int rr = 0; rr < 16; ++rr) {
            const int il = sub * 32 + acc_row(rr, grp);     // query row inside the tile
            float p = __builtin_amdgcn_exp2f(__fmaf_rn(s[rr], c2, -stat[il]));
            if (ji > i0 + il) p = 0.f;
            s[rr] = p;
            dp[rr] = p * (dp[rr] - stat[TILE + il]);
          }
        } else {
#pragma unroll
          for (int rr = 0; rr < 16; ++rr) {
            const int il = sub * 32 + acc_row(rr, grp);
            const float p = __builtin_amdgcn_exp2f(__fmaf_rn(s[rr], c2, -stat[il]));
            s[rr] = p;
            dp[rr] = p * (dp[rr] - stat[TILE + il]);
          }
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const bf16x8 pf = pack_frag(s, ks), dsf = pack_frag(dp, ks);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt) {
            dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(Okm, sub * 32 + ks * 16, dt * 32), pf,
                                                             dv[dt], 0, 0, 0);
            dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(Qkm, sub * 32 + ks * 16, dt * 32), dsf,
                                                             dk[dt], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();           // everyone is done reading this tile
    if (it + 1 < nit) park();
    __syncthreads();
  }
  if (!active) return;
  store_owned<DH>(dk, scale, dqkv + (tok0 + j0) * ld + d + h * DH, ld);
  store_owned<DH>(dv, 1.0f, dqkv + (tok0 + j0) * ld + 2 * d + h * DH, ld);
  if (colpart) {   // partial row (sequence, 32-key block) of the k and v thirds of the qkv bias gradient
    float* prow = colpart + ((tok0 + j0) / WROWS) * ld;
    colsum_owned<DH>(dk, scale, prow + d + h * DH);
    colsum_owned<DH>(dv, 1.0f, prow + 2 * d + h * DH);
  }
}

// ----------------------------------------------------------------------------------------
// backward, part 1: dQ, and D = rowsum(dO * O).  A wave owns 32 queries (lane = query); keys stream.
// ----------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_bwd_q_kernel(const uint16_t* __restrict__ qkv, int64_t ld,
                                                              const uint16_t* __restrict__ dout, int64_t ldo,
                                                              const uint16_t* __restrict__ outp,
                                                              const float* __restrict__ lse2,
                                                              float* __restrict__ Dv,
                                                              uint16_t* __restrict__ dqkv, int S, int d, int H,
                                                              int nseq, float c2, float scale,
                                                              float* __restrict__ colpart) {
  extern __shared__ __align__(16) char smem[];
  char* Kkc = smem;                         // K tile, k-contiguous (S^T = K Q^T)
  char* Kkm = Kkc + L<DH>::KC_BYTES;        // K tile, transpose-read (dQ^T = K^T dS^T)
  char* Vkc = Kkm + L<DH>::KM_BYTES;        // V tile, k-contiguous (dP^T = V dO^T)

  const int nblk = (S + BROWS - 1) / BROWS;
  int rank, h, b;
  attn_block(H, nseq, rank, h, b);
  const int qb = nblk - 1 - rank;
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, grp = l >> 5;
  const int q0 = qb * BROWS + wave * WROWS;
  const bool active = q0 < S;
  const int64_t tok0 = (int64_t)b * S;
  const uint16_t* Kg = qkv + tok0 * ld + d + h * DH;
  const uint16_t* Vg = qkv + tok0 * ld + 2 * d + h * DH;
  const int qi = q0 + (l & 31);

  bf16x8 qf[DH / 16], of[DH / 16];
  float lse_i = 0.f, D_i = 0.f;
  if (active) {
    load_owned<DH>(qf, qkv + (tok0 + q0) * ld + h * DH, ld);
    load_owned<DH>(of, dout + (tok0 + q0) * ldo + h * DH, ldo);
    lse_i = lse2[((int64_t)b * H + h) * S + qi];
    // D_i = sum_dh dO[i,dh] * O[i,dh]: the wave holds its rows of dO as fragments already; the
    // rows of O come in the same layout.  Stored for the dK/dV kernel, which runs after this one.
    bf16x8 oo[DH / 16];
    load_owned<DH>(oo, outp + (tok0 + q0) * ldo + h * DH, ldo);
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      const u32x4 a = __builtin_bit_cast(u32x4, oo[kk]), g = __builtin_bit_cast(u32x4, of[kk]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        D_i = __fmaf_rn(__uint_as_float(a[e] << 16), __uint_as_float(g[e] << 16), D_i);
        D_i = __fmaf_rn(__uint_as_float(a[e] & 0xFFFF0000u), __uint_as_float(g[e] & 0xFFFF0000u), D_i);
      }
    }
    D_i += __shfl_xor(D_i, 32, 64);
    if (grp == 0) Dv[((int64_t)b * H + h) * S + qi] = D_i;
  }
  f32x16 dq[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) dq[dt] = zero16();

  const int nkt = min(S, (qb + 1) * BROWS) / TILE;
  u32x4 rk[L<DH>::CHUNKS], rv[L<DH>::CHUNKS];
  auto fetch = [&](int kt) {
    g2r<DH>(rk, Kg + (int64_t)kt * TILE * ld, ld);
    g2r<DH>(rv, Vg + (int64_t)kt * TILE * ld, ld);
  };
  auto park = [&]() {
    r2s<DH, L<DH>::PKC>(rk, Kkc); r2s<DH, L<DH>::PKM>(rk, Kkm);
    r2s<DH, L<DH>::PKC>(rv, Vkc);
  };
  fetch(0); park();
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const int k0 = kt * TILE;
    if (kt + 1 < nkt) fetch(kt + 1);
    if (active && k0 <= q0 + WROWS - 1) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int ks0 = k0 + sub * 32;
        if (ks0 > q0 + WROWS - 1) continue;
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int kk = 0; kk < DH / 16; ++kk) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<DH>(Kkc, sub * 32, kk), qf[kk], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<DH>(Vkc, sub * 32, kk), of[kk], dp, 0, 0, 0);
        }
        const bool diag = ks0 + 31 > q0;                  // wave-uniform: only diagonal tiles mask
        if (diag) {
#pragma unroll
          for (int rr = 0; rr < 16; ++rr) {
            float p = __builtin_amdgcn_exp2f(__fmaf_rn(s[rr], c2, -lse_i));
            if (ks0 + acc_row(rr, grp) > qi) p = 0.f;
            dp[rr] = p * (dp[rr] - D_i);
          }
        } else {
#pragma unroll
          for (int rr = 0; rr < 16; ++rr)
            dp[rr] = __builtin_amdgcn_exp2f(__fmaf_rn(s[rr], c2, -lse_i)) * (dp[rr] - D_i);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const bf16x8 dsf = pack_frag(dp, ks);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt)
            dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(Kkm, sub * 32 + ks * 16, dt * 32), dsf,
                                                             dq[dt], 0, 0, 0);
        }
      }
    }
    __syncthreads();           // everyone is done reading this tile
    if (kt + 1 < nkt) park();
    __syncthreads();
  }
  if (!active) return;
  store_owned<DH>(dq, scale, dqkv + (tok0 + q0) * ld + h * DH, ld);
  if (colpart) colsum_owned<DH>(dq, scale, colpart + ((tok0 + q0) / WROWS) * ld + h * DH);   // the q third
}

template <typename K>
rv_status set_smem(K kern, int bytes) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? RV_OK : RV_E_DEVICE;
}

bool shape_ok(int mb, int S, int d, int H) {
  if (mb < 1 || H < 1 || d % H) return false;
  const int dh = d / H;
  return (dh == 64 || dh == 128) && S >= TILE && S % TILE == 0;
}

}  // namespace

rv_status rv_attn_fwd(const uint16_t* qkv, uint16_t* out, float* lse2, int mb, int S, int d, int H,
                      hipStream_t st) {
  if (!qkv || !out || !lse2 || !shape_ok(mb, S, d, H)) return RV_E_INVAL;
  const int dh = d / H;
  const float c2 = 1.4426950408889634f / sqrtf((float)dh);
  const int nwg = ((S + BROWS - 1) / BROWS) * H * mb;
  dim3 grid(nwg);
  if (dh == 64) {
    constexpr int smem = 2 * (L<64>::KC_BYTES + L<64>::KM_BYTES);
    RV_TRY(set_smem(attn_fwd_kernel<64>, smem));
    hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(kThreads), smem, st, qkv, (int64_t)3 * d, out, (int64_t)d,
                       lse2, S, d, H, mb, c2);
  } else {
    constexpr int smem = 2 * (L<128>::KC_BYTES + L<128>::KM_BYTES);
    RV_TRY(set_smem(attn_fwd_kernel<128>, smem));
    hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(kThreads), smem, st, qkv, (int64_t)3 * d, out,
                       (int64_t)d, lse2, S, d, H, mb, c2);
  }
  return rv_launch_status();
}

int rv_attn_colsum_parts(int mb, int S) { return mb * (S / WROWS); }

rv_status rv_attn_bwd(const uint16_t* qkv, const uint16_t* out, const uint16_t* dout, const float* lse2,
                      float* Dbuf, uint16_t* dqkv, int mb, int S, int d, int H, hipStream_t st, float* colpart) {
  if (!qkv || !out || !dout || !lse2 || !Dbuf || !dqkv || !shape_ok(mb, S, d, H)) return RV_E_INVAL;
  const int dh = d / H;
  const float scale = 1.0f / sqrtf((float)dh);
  const float c2 = 1.4426950408889634f * scale;
  const int nwg = ((S + BROWS - 1) / BROWS) * H * mb;
  dim3 grid(nwg);
  if (dh == 64) {
    constexpr int s1 = 2 * (L<64>::KC_BYTES + L<64>::KM_BYTES) + 2 * TILE * 4;
    constexpr int s2 = 2 * L<64>::KC_BYTES + L<64>::KM_BYTES;
    RV_TRY(set_smem(attn_bwd_kv_kernel<64>, s1)); RV_TRY(set_smem(attn_bwd_q_kernel<64>, s2));
    hipLaunchKernelGGL(attn_bwd_q_kernel<64>, grid, dim3(kThreads), s2, st, qkv, (int64_t)3 * d, dout, (int64_t)d,
                       out, lse2, Dbuf, dqkv, S, d, H, mb, c2, scale, colpart);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<64>, grid, dim3(kThreads), s1, st, qkv, (int64_t)3 * d, dout, (int64_t)d,
                       lse2, Dbuf, dqkv, S, d, H, mb, c2, scale, colpart);
  } else {
    constexpr int s1 = 2 * (L<128>::KC_BYTES + L<128>::KM_BYTES) + 2 * TILE * 4;
    constexpr int s2 = 2 * L<128>::KC_BYTES + L<128>::KM_BYTES;
    RV_TRY(set_smem(attn_bwd_kv_kernel<128>, s1)); RV_TRY(set_smem(attn_bwd_q_kernel<128>, s2));
    hipLaunchKernelGGL(attn_bwd_q_kernel<128>, grid, dim3(kThreads), s2, st, qkv, (int64_t)3 * d, dout, (int64_t)d,
                       out, lse2, Dbuf, dqkv, S, d, H, mb, c2, scale, colpart);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<128>, grid, dim3(kThreads), s1, st, qkv, (int64_t)3 * d, dout, (int64_t)d,
                       lse2, Dbuf, dqkv, S, d, H, mb, c2, scale, colpart);
  }
  return rv_launch_status();
}

extern "C" rv_status rv_k_attention_fwd(const void* qkv, void* out, float* lse2, int microbatch, int seq,
                                        int d_model, int n_heads, void* stream) {
  return rv_attn_fwd((const uint16_t*)qkv, (uint16_t*)out, lse2, microbatch, seq, d_model, n_heads,
                     (hipStream_t)stream);
}

extern "C" rv_status rv_k_attention_bwd(const void* qkv, const void* out, const void* dout, const float* lse2,
                                        float* dscratch, void* dqkv, int microbatch, int seq, int d_model,
                                        int n_heads, void* stream) {
  return rv_attn_bwd((const uint16_t*)qkv, (const uint16_t*)out, (const uint16_t*)dout, lse2, dscratch,
                     (uint16_t*)dqkv, microbatch, seq, d_model, n_heads, (hipStream_t)stream);
}

// ---- the backward for callers that cannot allocate ---------------------------------------
// The per-row term D = rowsum(dO * O) that the two backward kernels exchange lives in a
// file-scope device array instead of a caller workspace.  Every GPU holds its own copy of
// the array; its address on a device is looked up once, with that device current.
namespace {
constexpr int kStaticRows = 262144;   // 1 MiB: microbatch * n_heads * seq may not exceed this
static __device__ __align__(256) float scratch[kStaticRows];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};   // per device, filled on first use
std::mutex g_scratch_mu;

rv_status static_scratch(float** out) {
  int dev = -1;
  RV_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RV_E_INVAL;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    RV_HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return RV_E_DEVICE;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RV_OK;
}
}  // namespace

extern "C" rv_status rv_k_attention_bwd_static(const void* qkv, const void* out, const void* dout,
                                               const float* lse2, void* dqkv, int microbatch, int seq,
                                               int d_model, int n_heads, void* stream) {
  if (microbatch < 1 || seq < 1 || n_heads < 1 ||
      (int64_t)microbatch * n_heads * seq > (int64_t)kStaticRows)
    return RV_E_INVAL;   // beyond the fixed scratch
  float* D = nullptr;
  RV_TRY(static_scratch(&D));
  // every row of D that the second kernel reads is written by the first one in this call:
  // nothing of the previous call's contents is used, so nothing has to be cleared
  return rv_attn_bwd((const uint16_t*)qkv, (const uint16_t*)out, (const uint16_t*)dout, lse2, D,
                     (uint16_t*)dqkv, microbatch, seq, d_model, n_heads, (hipStream_t)stream);
}
