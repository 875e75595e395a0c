// Decoder stage: L pre-LayerNorm transformer blocks as one peer's forward_pass and its
// exact gradient at the stashed weight version (paper Alg. 1; Eq. 2).  Host-side
// sequencing only; the work is in gemm_bf16.hip, attention.hip and norm.hip.
//
//   u  = LN1(x);  qkv = u Wqkv + bqkv;  a = CausalSoftmax(q k^T / sqrt(dh)) v
//   x1 = x + a Wo + bo;   v2 = LN2(x1);  z = v2 W1 + b1;  g = GELU(z);  y = x1 + g W2 + b2
//
// The residual stream (x, x1, y) and its gradient are fp32 inside the stage; matrix
// product operands are bf16.  Per microbatch and block the stash keeps x, x1 (fp32), the
// LN statistics, u, qkv, a, v2, z, g (bf16) and the softmax log-sums: everything the
// backward reads, so nothing is recomputed except the attention probabilities.
#include <new>
#include "internal.h"

namespace {

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct DecPlan {
  int L, d, H, f, S, mb, T;
  // element offsets inside one block's parameters (same in the fp32 master and the bf16 version)
  size_t ln1g, ln1b, wqkv, bqkv, wo, bo, ln2g, ln2b, w1, b1, w2, b2, per_block;
  // byte offsets inside one block's stash
  size_t s_x, s_m1, s_r1, s_u, s_qkv, s_a, s_lse, s_x1, s_m2, s_r2, s_v2, s_z, s_g, blk_bytes;
  // byte offsets inside the work buffer
  // (dy: three buffers, dx1 / dz / dqkv: two, so a block's weight-gradient products can run
  // beside the next block)
  size_t w_dres, w_dy[3], w_dx1_16[2], w_dtmp, w_dz[2], w_dqkv[2], w_D, w_part_ln[2][2], w_part_dy, w_part_dz[2],
      w_part_qkv[2], w_ytmp;
};

}  // namespace

rv_status rv_dec_plan(rv_stage* s) {
  const int64_t d = s->dims[0], H = s->dims[1], f = s->dims[2], S = s->dims[3];
  if (d < 64 || d > 4096 || d % 64 || H < 1 || d % H || f < 64 || f % 64 || f > (1 << 16) || S < 64 ||
      S % 64 || S > (1 << 16))
    return RV_E_INVAL;
  const int64_t dh = d / H;
  if (dh != 64 && dh != 128) return RV_E_INVAL;
  if ((int64_t)s->microbatch * S > (1 << 24)) return RV_E_INVAL;
  DecPlan* p = new (std::nothrow) DecPlan();
  if (!p) return RV_E_NOMEM;
  s->impl = p;
  p->L = s->n_layers; p->d = (int)d; p->H = (int)H; p->f = (int)f; p->S = (int)S; p->mb = s->microbatch;
  p->T = p->mb * p->S;
  size_t o = 0;
  p->ln1g = o; o += d; p->ln1b = o; o += d;
  p->wqkv = o; o += (size_t)d * 3 * d; p->bqkv = o; o += 3 * d;
  p->wo = o; o += (size_t)d * d; p->bo = o; o += d;
  p->ln2g = o; o += d; p->ln2b = o; o += d;
  p->w1 = o; o += (size_t)d * f; p->b1 = o; o += f;
  p->w2 = o; o += (size_t)f * d; p->b2 = o; o += d;
  p->per_block = o;
  s->P = o * p->L;
  const size_t T = p->T;
  size_t b = 0;
  p->s_x = b; b += align_up(T * d * 4);
  p->s_m1 = b; b += align_up(T * 4); p->s_r1 = b; b += align_up(T * 4);
  p->s_u = b; b += align_up(T * d * 2);
  p->s_qkv = b; b += align_up(T * 3 * d * 2);
  p->s_a = b; b += align_up(T * d * 2);
  p->s_lse = b; b += align_up(T * H * 4);
  p->s_x1 = b; b += align_up(T * d * 4);
  p->s_m2 = b; b += align_up(T * 4); p->s_r2 = b; b += align_up(T * 4);
  p->s_v2 = b; b += align_up(T * d * 2);
  p->s_z = b; b += align_up(T * f * 2);
  p->s_g = b; b += align_up(T * f * 2);
  p->blk_bytes = b;
  s->slot_bytes = b * p->L;
  size_t w = 0;
  p->w_dres = w; w += align_up(T * d * 4);
  for (size_t& o : p->w_dy) { o = w; w += align_up(T * d * 2); }
  for (size_t& o : p->w_dx1_16) { o = w; w += align_up(T * d * 2); }
  p->w_dtmp = w; w += align_up(T * d * 2);
  for (size_t& o : p->w_dz) { o = w; w += align_up(T * f * 2); }
  for (size_t& o : p->w_dqkv) { o = w; w += align_up(T * 3 * d * 2); }
  p->w_D = w; w += align_up(T * H * 4);
  const size_t part_ln = (size_t)rv_ln_bwd_parts(p->T, d) * 3 * d;
  for (auto& pair : p->w_part_ln)
    for (size_t& o : pair) { o = w; w += align_up(part_ln * 4); }
  // partial rows of the bias gradients: of the arriving gradient (32-row blocks), of dz (one per tile
  // row of the product that makes it, at least 128 rows) and of dqkv (32-token blocks)
  p->w_part_dy = w; w += align_up((size_t)rv_widen_parts(p->T) * d * 4);
  for (size_t& o : p->w_part_dz) { o = w; w += align_up((size_t)((T + 127) / 128) * f * 4); }
  for (size_t& o : p->w_part_qkv) { o = w; w += align_up((size_t)rv_attn_colsum_parts(p->mb, p->S) * 3 * d * 4); }
  p->w_ytmp = w; w += align_up(T * d * 4);
  s->work_bytes = w;
  return RV_OK;
}

void rv_dec_free(rv_stage* s) {
  delete (DecPlan*)s->impl;
  s->impl = nullptr;
}

namespace {

rv_status gemm(int sharing, hipStream_t st, const void* A, int64_t lda, int akm, const void* B, int64_t ldb, int bkm, int M,
               int N, int K, int epi, void* out, int64_t ldo, void* out2 = nullptr, const void* bias = nullptr,
               const float* resid = nullptr, const void* zin = nullptr, float* colpart = nullptr,
               int* colpart_rows = nullptr) {
  rv_gemm_args g;
  g.colpart = colpart;
  g.sharing = sharing;
  g.A = (const uint16_t*)A; g.lda = lda; g.a_kmajor = akm;
  g.B = (const uint16_t*)B; g.ldb = ldb; g.b_kmajor = bkm;
  g.M = M; g.N = N; g.K = K; g.epi = epi; g.out = out; g.ldo = ldo; g.out2 = out2;
  g.bias = (const uint16_t*)bias; g.resid = resid; g.ldr = ldo; g.zin = (const uint16_t*)zin;
  const rv_status rc = rv_gemm_bf16(g, st);
  if (colpart_rows) *colpart_rows = g.colpart_rows;
  return rc;
}

}  // namespace

rv_status rv_dec_forward(rv_stage* s, rv_slot& slot, const void* in, void* out) {
  const DecPlan& p = *(const DecPlan*)s->impl;
  const uint16_t* wv = (const uint16_t*)s->ver[slot.ver];
  hipStream_t st = s->st;
  const int T = p.T, d = p.d, f = p.f;
  const int sh = s->in_step ? 2 : 0;   // in a step the backward chain is the longer one
  for (int l = 0; l < p.L; ++l) {
    const uint16_t* w = wv + (size_t)l * p.per_block;
    char* sb = slot.base + (size_t)l * p.blk_bytes;
    float* x = (float*)(sb + p.s_x);
    float* x1 = (float*)(sb + p.s_x1);
    uint16_t* u = (uint16_t*)(sb + p.s_u);
    uint16_t* qkv = (uint16_t*)(sb + p.s_qkv);
    uint16_t* a = (uint16_t*)(sb + p.s_a);
    uint16_t* v2 = (uint16_t*)(sb + p.s_v2);
    uint16_t* z = (uint16_t*)(sb + p.s_z);
    uint16_t* g = (uint16_t*)(sb + p.s_g);
    if (l == 0)
      RV_TRY(rv_ln_fwd(in, 1, x, w + p.ln1g, w + p.ln1b, u, (float*)(sb + p.s_m1), (float*)(sb + p.s_r1), T, d,
                       s->ln_eps, st));
    else
      RV_TRY(rv_ln_fwd(x, 0, nullptr, w + p.ln1g, w + p.ln1b, u, (float*)(sb + p.s_m1), (float*)(sb + p.s_r1), T,
                       d, s->ln_eps, st));
    RV_TRY(gemm(sh, st, u, d, 0, w + p.wqkv, 3 * d, 1, T, 3 * d, d, RV_EPI_BF16_BIAS, qkv, 3 * d, nullptr, w + p.bqkv));
    RV_TRY(rv_attn_fwd(qkv, a, (float*)(sb + p.s_lse), p.mb, p.S, d, p.H, st));
    RV_TRY(gemm(sh, st, a, d, 0, w + p.wo, d, 1, T, d, d, RV_EPI_F32_BIAS_RESID, x1, d, nullptr, w + p.bo, x));
    RV_TRY(rv_ln_fwd(x1, 0, nullptr, w + p.ln2g, w + p.ln2b, v2, (float*)(sb + p.s_m2), (float*)(sb + p.s_r2), T, d,
                     s->ln_eps, st));
    RV_TRY(gemm(sh, st, v2, d, 0, w + p.w1, f, 1, T, f, d, RV_EPI_BF16_BIAS_GELU, z, f, g, w + p.b1));
    if (l + 1 < p.L) {
      float* xn = (float*)(slot.base + (size_t)(l + 1) * p.blk_bytes + p.s_x);
      RV_TRY(gemm(sh, st, g, f, 0, w + p.w2, d, 1, T, d, f, RV_EPI_F32_BIAS_RESID, xn, d, nullptr, w + p.b2, x1));
    } else {
      RV_TRY(gemm(sh, st, g, f, 0, w + p.w2, d, 1, T, d, f, RV_EPI_F32_BIAS_RESID_BF16, s->work + p.w_ytmp, d, out,
                  w + p.b2, x1));
    }
  }
  return RV_OK;
}

rv_status rv_dec_backward(rv_stage* s, rv_slot& slot, const void* grad_out, void* grad_in) {
  const DecPlan& p = *(const DecPlan*)s->impl;
  const uint16_t* wv = (const uint16_t*)s->ver[slot.ver];
  hipStream_t st = s->st;
  const int T = p.T, d = p.d, f = p.f;
  const int sh = s->in_step ? 1 : 0;
  float* dres = (float*)(s->work + p.w_dres);
  uint16_t* dtmp = (uint16_t*)(s->work + p.w_dtmp);
  float* Dbuf = (float*)(s->work + p.w_D);
  const int ln_parts = rv_ln_bwd_parts(T, d);
  // fused update (plain Eq. 2): every kernel that completes a parameter gradient applies it at once
  // to the fp32 master and writes the bf16 rounding into the new weight version `vdst`
  uint16_t* vdst = s->fused ? (uint16_t*)s->ver[s->upd_dst] : nullptr;
  rv_reduce_update ru;
  ru.eta = s->eta; ru.store = s->keep_grad;
  auto upd = [&](float* const* dst, int n) -> const rv_reduce_update* {
    if (!s->fused) return nullptr;
    for (int k = 0; k < n; ++k) {
      const size_t off = (size_t)(dst[k] - s->grad);
      ru.w[k] = s->master + off; ru.ver[k] = vdst + off;
    }
    return &ru;
  };

  // Everything that only feeds the parameter gradient - the four weight-gradient products of a
  // block, the reductions behind the bias and LayerNorm gradients, the block's delayed update -
  // is side work: nothing in the chain dy -> dx that the block below waits for reads it.  It
  // goes to a stream of its own and runs beside the next block's chain (measured step time
  // against issuing it in line: config 2 -7 %, config 3 -1 %, config 5 -5 %).  Buffers that
  // side work reads alternate between blocks (dy: in threes, since block l-1 writes the dy of
  // block l-2 while the side work of block l still reads its own).
  hipStream_t ws = s->wgs;
  auto side_begin = [&]() -> rv_status {
    RV_HIP_TRY(hipEventRecord(s->ev_wg_ready, st));
    RV_HIP_TRY(hipStreamWaitEvent(ws, s->ev_wg_ready, 0));
    return RV_OK;
  };

  // gradient of the last block's output: fp32 copy for the residual path, bf16 as operand
  // (summed over tokens it is also the gradient of the last block's b2: partial sums on the way)
  float* part_dy = (float*)(s->work + p.w_part_dy);
  RV_TRY(rv_widen_colsum((const uint16_t*)grad_out, dres, part_dy, T, d, st));
  const uint16_t* dres16 = (const uint16_t*)grad_out;
  {
    float* out = s->grad + (size_t)(p.L - 1) * p.per_block + p.b2;
    RV_TRY(side_begin());
    RV_TRY(rv_reduce_rows(part_dy, rv_widen_parts(T), d, d, out, ws, upd(&out, 1)));
  }
  // When the four weight-gradient products of a block go to the side stream.  Launch points:
  // 0 behind the GELU' product (dz exists: dW2 and dW1 can run), 1 behind the second LayerNorm's
  // backward (dx1 exists: dWo), 2 behind the attention backward (dqkv exists: all four).  One
  // launch of all four at point 2 is the least launch work; going out earlier puts the products
  // beside the chain's LayerNorm and attention kernels instead of beside its next products.
  // Measured step time against the single launch, tiles of 256 x 256 on 256 CUs:
  //   dW2 + dW1 at point 0, dWo + dWqkv at point 2:  -4.7 % where they are 512 and 256 tiles
  //   (d 2048, ffn 8192), 0 % at 350 and 182 tiles (d 1600, ffn 6400), +1.3 % at 128 and 64 tiles
  //   (d 1024, ffn 4096);
  //   dWo on its own at point 1 as well:  -2.8 %, -1.2 %, +7 % in the same order.
  // So: the feed-forward pair goes out early when it fills the chip at least once, and dWo leaves
  // dWqkv only when the two together are not a whole number of rounds anyway.
  const int kCUs = 256;
  auto tiles = [](int M, int N) { return ((M + 255) / 256) * ((N + 255) / 256); };
  const int n_ffn = 2 * tiles(d, f), n_o = tiles(d, d), n_qkv = tiles(d, 3 * d);
  int wg_pos[4] = {2, 2, 2, 2};   // dW2, dW1, dWo, dWqkv
  if (n_ffn >= kCUs) {
    wg_pos[0] = wg_pos[1] = 0;
    if ((n_o + n_qkv) % kCUs != 0) wg_pos[2] = 1;
  }
  for (int l = p.L - 1; l >= 0; --l) {
    const int par = l & 1;
    // block l may overwrite what the side work of block l+2 read only after that is done
    if (l + 2 < p.L) RV_HIP_TRY(hipStreamWaitEvent(st, s->ev_wg_done[par], 0));
    uint16_t* dx1_16 = (uint16_t*)(s->work + p.w_dx1_16[par]);   // bf16 dx1 of this block
    uint16_t* dz = (uint16_t*)(s->work + p.w_dz[par]);
    uint16_t* dqkv = (uint16_t*)(s->work + p.w_dqkv[par]);
    uint16_t* dy_below = (uint16_t*)(s->work + p.w_dy[(l + 2) % 3]);   // = slot (l-1) mod 3
    float* part2 = (float*)(s->work + p.w_part_ln[par][0]);      // LayerNorm 2 / 1 partial sums
    float* part1 = (float*)(s->work + p.w_part_ln[par][1]);
    const uint16_t* w = wv + (size_t)l * p.per_block;
    float* gl = s->grad + (size_t)l * p.per_block;
    const char* sb = slot.base + (size_t)l * p.blk_bytes;
    const float* x = (const float*)(sb + p.s_x);
    const float* x1 = (const float*)(sb + p.s_x1);
    const uint16_t* u = (const uint16_t*)(sb + p.s_u);
    const uint16_t* qkv = (const uint16_t*)(sb + p.s_qkv);
    const uint16_t* a = (const uint16_t*)(sb + p.s_a);
    const uint16_t* v2 = (const uint16_t*)(sb + p.s_v2);
    const uint16_t* z = (const uint16_t*)(sb + p.s_z);
    const uint16_t* g = (const uint16_t*)(sb + p.s_g);
    rv_gemm_args wg[4];
    // the weight-gradient products whose launch point is `pos` go out as one grouped launch
    auto side_launch = [&](int pos) -> rv_status {
      rv_gemm_args grp[4];
      int n = 0;
      for (int k = 0; k < 4; ++k)
        if (wg_pos[k] == pos) grp[n++] = wg[k];
      if (!n) return RV_OK;
      if (s->prof_on) {   // measurement aid: bracket the launch with events on its own stream
        hipEvent_t e0 = nullptr, e1 = nullptr;
        RV_HIP_TRY(hipEventCreate(&e0));
        s->prof_ev.push_back(e0);
        RV_HIP_TRY(hipEventCreate(&e1));
        s->prof_ev.push_back(e1);
        RV_HIP_TRY(hipEventRecord(e0, ws));
        RV_TRY(rv_gemm_wgrad_grouped(grp, n, ws));
        RV_HIP_TRY(hipEventRecord(e1, ws));
        return RV_OK;
      }
      return rv_gemm_wgrad_grouped(grp, n, ws);
    };
    auto wgrad = [&](int k, const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int M, int N, float* out) {
      wg[k].A = A; wg[k].lda = lda; wg[k].a_kmajor = 1; wg[k].B = B; wg[k].ldb = ldb; wg[k].b_kmajor = 1;
      wg[k].M = M; wg[k].N = N; wg[k].K = T; wg[k].epi = RV_EPI_F32; wg[k].out = out; wg[k].ldo = N;
      if (s->fused) {   // Eq. 2 in the product's epilogue: master and new weight version at the same offset
        const size_t off = (size_t)(out - s->grad);
        wg[k].upd_w = s->master + off; wg[k].upd_ver = vdst + off; wg[k].upd_eta = s->eta;
        wg[k].store_out = s->keep_grad;
      }
    };
    // feed-forward half
    wgrad(0, g, f, dres16, d, f, d, gl + p.w2);                                                      // dW2 = g^T dy
    // dz = (dy W2^T) * GELU'(z); its column sums (the b1 gradient) leave the same epilogue as partial rows
    float* part_dz = (float*)(s->work + p.w_part_dz[par]);
    int dz_parts = 0;
    RV_TRY(gemm(sh, st, dres16, d, 0, w + p.w2, d, 0, T, f, d, RV_EPI_BF16_DGELU, dz, f, nullptr, nullptr, nullptr, z,
                part_dz, &dz_parts));
    wgrad(1, v2, d, dz, f, d, f, gl + p.w1);                                                         // dW1 = v2^T dz
    RV_TRY(side_begin());
    RV_TRY(side_launch(0));
    {
      float* out = gl + p.b1;
      RV_TRY(rv_reduce_rows(part_dz, dz_parts, f, f, out, ws, upd(&out, 1)));
    }
    RV_TRY(gemm(sh, st, dz, f, 0, w + p.w1, f, 0, T, d, f, RV_EPI_BF16, dtmp, d));                       // dv2 = dz W1^T
    RV_TRY(rv_ln_bwd(dtmp, x1, (const float*)(sb + p.s_m2), (const float*)(sb + p.s_r2), w + p.ln2g, dres, dres,
                     dx1_16, part2, T, d, st));
    {
      const float* src[3] = {part2, part2 + d, part2 + 2 * d};
      float* dst[3] = {gl + p.ln2g, gl + p.ln2b, gl + p.bo};                                         // dbo = sum dx1
      RV_TRY(side_begin());
      RV_TRY(rv_reduce_rows_multi(src, dst, 3, ln_parts, 3 * (int64_t)d, d, ws, upd(dst, 3)));
    }
    // attention half
    wgrad(2, a, d, dx1_16, d, d, d, gl + p.wo);                                                      // dWo = a^T dx1
    RV_TRY(side_launch(1));   // (the side stream already waits for the LayerNorm backward above)
    RV_TRY(gemm(sh, st, dx1_16, d, 0, w + p.wo, d, 0, T, d, d, RV_EPI_BF16, dtmp, d));                   // da = dx1 Wo^T
    // (the attention backward also leaves partial column sums of dqkv: the qkv bias gradient)
    float* part_qkv = (float*)(s->work + p.w_part_qkv[par]);
    RV_TRY(rv_attn_bwd(qkv, a, dtmp, (const float*)(sb + p.s_lse), Dbuf, dqkv, p.mb, p.S, d, p.H, st, part_qkv));
    wgrad(3, u, d, dqkv, 3 * d, d, 3 * d, gl + p.wqkv);                                              // dWqkv = u^T dqkv
    RV_TRY(side_begin());
    RV_TRY(side_launch(2));
    {
      float* out = gl + p.bqkv;
      RV_TRY(rv_reduce_rows(part_qkv, rv_attn_colsum_parts(p.mb, p.S), 3 * d, 3 * d, out, ws, upd(&out, 1)));
    }
    RV_TRY(gemm(sh, st, dqkv, 3 * d, 0, w + p.wqkv, 3 * d, 0, T, d, 3 * d, RV_EPI_BF16, dtmp, d));       // du
    uint16_t* dx16 = l == 0 ? (uint16_t*)grad_in : dy_below;
    RV_TRY(rv_ln_bwd(dtmp, x, (const float*)(sb + p.s_m1), (const float*)(sb + p.s_r1), w + p.ln1g, dres, dres, dx16,
                     part1, T, d, st));
    {
      // the residual gradient leaving this block is dy of the block below: its b2 gradient
      const float* src[3] = {part1, part1 + d, part1 + 2 * d};
      float* dst[3] = {gl + p.ln1g, gl + p.ln1b, l > 0 ? s->grad + (size_t)(l - 1) * p.per_block + p.b2 : nullptr};
      RV_TRY(side_begin());
      RV_TRY(rv_reduce_rows_multi(src, dst, l > 0 ? 3 : 2, ln_parts, 3 * (int64_t)d, d, ws, upd(dst, l > 0 ? 3 : 2)));
    }
    // every gradient of block l is complete behind this point of `ws` (its b2 gradient came
    // from the block above); unless the epilogues above have applied it already, the delayed
    // update of the block follows at once
    if (!s->fused) RV_TRY(rv_stage_update_range(s, (size_t)l * p.per_block, p.per_block, ws));
    RV_HIP_TRY(hipEventRecord(s->ev_wg_done[par], ws));
    dres16 = dy_below;               // dy of the block below
  }
  // the caller's stream (and with it the update) continues behind the last side work
  RV_HIP_TRY(hipStreamWaitEvent(st, s->ev_wg_done[0], 0));
  if (p.L > 1) RV_HIP_TRY(hipStreamWaitEvent(st, s->ev_wg_done[1], 0));
  return RV_OK;
}
