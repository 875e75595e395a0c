// Internal interfaces between the library's translation units (not part of the ABI).
#pragma once
#include <vector>
#include "common.h"

// ---- update.hip ------------------------------------------------------------------
// copy_kind: 0 none, 1 bf16 bits, 2 fp32
rv_status rv_launch_update(float* w, const float* g, size_t n, float eta, void* copy, int copy_kind,
                           hipStream_t st);
rv_status rv_launch_update_momentum(float* w, const float* g, float* v, size_t n, float eta, float mu, float wd,
                                    void* copy, int copy_kind, hipStream_t st);
rv_status rv_launch_accumulate(float* acc, const float* g, size_t n, bool first, hipStream_t st);
rv_status rv_launch_publish(const float* w, size_t n, void* copy, int copy_kind, hipStream_t st);

// ---- gemm_bf16.hip ----------------------------------------------------------------
#include "../../include/rv_kernels.h"
struct rv_gemm_args {
  const uint16_t* A = nullptr; int64_t lda = 0; int a_kmajor = 0;
  const uint16_t* B = nullptr; int64_t ldb = 0; int b_kmajor = 0;
  int M = 0, N = 0, K = 0;
  int epi = 0;
  void* out = nullptr; int64_t ldo = 0;   // primary output [M, ldo]
  void* out2 = nullptr;                   // second output, same pitch (GELU value / bf16 copy)
  const uint16_t* bias = nullptr;         // bf16 [N]
  const float* resid = nullptr; int64_t ldr = 0;
  const uint16_t* zin = nullptr;          // bf16 [M, ldo] pre-activations for GELU'
  int tile = 0;                           // 0 = choose, 128 or 256 = force
  // who else is on the chip while this product runs (automatic tile choice only):
  //   0  nobody: shortest time of this launch alone
  //   1  the other streams of a stage step, and the launch is on the step's critical chain:
  //      the 256x256 tile as soon as it covers half the chip
  //   2  the same, off the critical chain: always the 256x256 tile (least CU time per flop)
  int sharing = 0;
  // weight-gradient products of the grouped launch only: the delayed update of Eq. 2 applied in
  // the epilogue.  upd_w = fp32 master tile base (same [M, ldo] layout as out), upd_ver = bf16
  // weight-version tile base; the gradient itself is stored to `out` only if store_out.
  // GELU' epilogue only: if given, fp32 [ceil(M / tile rows), ldo] partial column sums of the
  // output (the bias gradient of the Linear whose pre-activation gradient this is), one row per
  // tile row; the number of rows written comes back in colpart_rows
  float* colpart = nullptr;
  mutable int colpart_rows = 0;
  float* upd_w = nullptr;
  uint16_t* upd_ver = nullptr;
  float upd_eta = 0.f;
  bool store_out = true;
};
rv_status rv_gemm_bf16(const rv_gemm_args& g, hipStream_t st);
// up to RV_GEMM_GROUP_MAX weight-gradient products (both operands k-major, fp32 output) in one launch
#define RV_GEMM_GROUP_MAX 4
rv_status rv_stage_update_range(rv_stage* s, size_t off, size_t n, hipStream_t st);
rv_status rv_gemm_wgrad_grouped(const rv_gemm_args* gs, int count, hipStream_t st);

// ---- norm.hip ---------------------------------------------------------------------
rv_status rv_ln_fwd(const void* x, int x_is_bf16, float* xcopy, const uint16_t* gamma, const uint16_t* beta,
                    uint16_t* y, float* mean, float* rstd, int T, int d, float eps, hipStream_t st);
int rv_ln_bwd_parts(int T, int d);   // partial rows written by rv_ln_bwd (each 3*d floats)
rv_status rv_ln_bwd(const uint16_t* dy, const float* x, const float* mean, const float* rstd,
                    const uint16_t* gamma, const float* dres, float* dx, uint16_t* dx_bf16, float* part,
                    int T, int d, hipStream_t st);
// o fp32 [T,d] = a bf16 [T,d] widened, and part fp32 [rv_widen_parts(T), d] = column sums of a over
// blocks of 32 rows
int rv_widen_parts(int T);
rv_status rv_widen_colsum(const uint16_t* a, float* o, float* part, int T, int d, hipStream_t st);
// out_k[c] = sum_r src_k[r * pitch + c].  upd (may be null): per job the fp32 master vector and the
// bf16 weight-version vector the column sums update in place, w <- w - eta * sum (Eq. 2); with
// store = false the sums themselves are not written.
struct rv_reduce_update {
  float* w[4];
  uint16_t* ver[4];
  float eta;
  bool store;
};
rv_status rv_reduce_rows_multi(const float* const* src, float* const* out, int njobs, int R, int64_t pitch,
                               int N, hipStream_t st, const rv_reduce_update* upd = nullptr);
rv_status rv_reduce_rows(const float* part, int R, int64_t pitch, int N, float* out, hipStream_t st,
                         const rv_reduce_update* upd = nullptr);

// ---- attention.hip ----------------------------------------------------------------
rv_status rv_attn_fwd(const uint16_t* qkv, uint16_t* out, float* lse2, int mb, int S, int d, int H,
                      hipStream_t st);
// colpart (may be null): fp32 [mb*S/32, 3d] partial rows of the column sums of dqkv (the qkv
// bias gradient), one per (sequence, 32-token block); reduce with rv_reduce_rows
int rv_attn_colsum_parts(int mb, int S);
rv_status rv_attn_bwd(const uint16_t* qkv, const uint16_t* out, const uint16_t* dout, const float* lse2,
                      float* Dbuf, uint16_t* dqkv, int mb, int S, int d, int H, hipStream_t st,
                      float* colpart = nullptr);

// ---- stage bookkeeping -------------------------------------------------------------
struct rv_slot {
  bool live = false;
  int64_t mb = 0;
  int ver = -1;          // weight-version slot bound at forward time
  char* base = nullptr;  // activation stash of this microbatch
};

struct rv_stage {
  int kind = 0, dtype = 0, n_layers = 0, microbatch = 0, tau = 0;
  float eta = 0.f, ln_eps = 1e-5f;
  std::vector<int64_t> dims;
  hipStream_t st = nullptr;   // stream the next kernel is enqueued on (the caller's, or aux inside a step)
  hipStream_t aux = nullptr;  // second stream for the backward half of rv_stage_step
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  // third stream: the weight-gradient products of a decoder block run beside the next block's
  // input-gradient chain
  int upd_dst = -1;           // version slot the running backward publishes into
  bool in_step = false;       // inside rv_stage_step: forward and backward share the chip
  hipStream_t wgs = nullptr;
  hipEvent_t ev_wg_ready = nullptr, ev_wg_done[2] = {nullptr, nullptr};
  size_t P = 0;
  float* master = nullptr;  // [P] fp32
  float* grad = nullptr;    // [P] fp32, gradient of the last backward
  float* vel = nullptr;     // [P] fp32 momentum buffer (allocated by rv_stage_set_optimizer)
  float momentum = 0.f, weight_decay = 0.f;
  float* gacc = nullptr;    // [P] fp32 sum of the gradients of the current accumulation group
  int accum = 1, acc_count = 0;   // microbatches per update; backwards so far in the group
  bool defer = false;       // backward leaves its update pending (folded into the next cluster sync)
  bool keep_grad = false;   // decoder: also store the parameter gradient when the update is applied in the
                            // epilogues that produce it (rv_stage_keep_grad)
  bool fused = false;       // the running backward applies Eq. 2 in those epilogues
  bool grad_valid = false;  // `grad` holds the whole gradient of the last backward
  size_t ver_elem = 0;      // bytes per parameter in a version slot (2 or 4)
  std::vector<char*> ver;   // tau+2 version slots: one is always free of readers, so an update can be
                            // written piece by piece while the backward still reads its own version
  std::vector<int> ver_ref; // in-flight microbatches bound to each slot
  int cur = 0;              // slot holding the newest version
  std::vector<rv_slot> slots;
  size_t slot_bytes = 0;
  char* stash = nullptr;    // (tau+1) * slot_bytes
  char* work = nullptr;     // scratch shared by all calls of this stage
  size_t work_bytes = 0;
  void* impl = nullptr;     // kind-specific plan (offsets, shapes)
  // rv_cluster_sync_fork .. join: the version slot the averaging is writing on another stream
  // (-1: none), and the stage whose ev_sync_done closes it
  int sync_dst = -1;
  rv_stage* sync_owner = nullptr;
  hipEvent_t ev_sync_ready = nullptr, ev_sync_done = nullptr;
  // rv_stage_profile: event pairs around every launch of the block's grouped weight-gradient
  // product, on the stream it is launched on
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;   // start, stop, start, stop, ...
};

// ---- mlp.hip -----------------------------------------------------------------------
rv_status rv_mlp_plan(rv_stage* s);   // fills P, slot_bytes, work_bytes, impl
void rv_mlp_free(rv_stage* s);
rv_status rv_mlp_forward(rv_stage* s, rv_slot& slot, const void* in, void* out);
rv_status rv_mlp_backward(rv_stage* s, rv_slot& slot, const void* grad_out, void* grad_in);

// ---- decoder.hip -------------------------------------------------------------------
rv_status rv_dec_plan(rv_stage* s);
void rv_dec_free(rv_stage* s);
rv_status rv_dec_forward(rv_stage* s, rv_slot& slot, const void* in, void* out);
rv_status rv_dec_backward(rv_stage* s, rv_slot& slot, const void* grad_out, void* grad_in);
