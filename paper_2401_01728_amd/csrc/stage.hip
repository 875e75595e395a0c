// Stage object: one peer of the paper's Alg. 1.  Host-side bookkeeping only:
//   - the microbatch -> stash-slot map (at most tau+1 in flight: the paper's rule that a
//     sender waits until the receiver's buffer has room becomes RV_E_STASH_FULL),
//   - the ring of weight versions.  A forward binds the microbatch to the newest version; its
//     backward reads exactly that version (Eq. 2 takes the gradient at the parameters in force
//     during the forward); the update publishes a new version into a slot no in-flight
//     microbatch refers to.  tau+1 microbatches can be in flight, each bound to a version of
//     its own, so tau+2 slots are kept: the new version can then be written piece by piece, by
//     the kernels that produce the gradient, while the backward still reads its own.
// All device work is enqueued on the stage's stream by mlp.hip / decoder.hip / update.hip.
#include <new>
#include "internal.h"

namespace {

int find_slot(const rv_stage* s, int64_t mb) {
  for (size_t i = 0; i < s->slots.size(); ++i)
    if (s->slots[i].live && s->slots[i].mb == mb) return (int)i;
  return -1;
}

int copy_kind(const rv_stage* s) { return s->dtype == RV_BF16 ? 1 : 2; }

void free_all(rv_stage* s) {
  if (!s) return;
  if (s->kind == RV_MLP) rv_mlp_free(s); else rv_dec_free(s);
  for (hipEvent_t ev : s->prof_ev) if (ev) (void)hipEventDestroy(ev);
  if (s->ev_sync_ready) (void)hipEventDestroy(s->ev_sync_ready);
  if (s->ev_sync_done) (void)hipEventDestroy(s->ev_sync_done);
  if (s->ev_fork) (void)hipEventDestroy(s->ev_fork);
  if (s->ev_join) (void)hipEventDestroy(s->ev_join);
  if (s->aux) (void)hipStreamDestroy(s->aux);
  if (s->ev_wg_ready) (void)hipEventDestroy(s->ev_wg_ready);
  for (hipEvent_t ev : s->ev_wg_done) if (ev) (void)hipEventDestroy(ev);
  if (s->wgs) (void)hipStreamDestroy(s->wgs);
  if (s->master) (void)hipFree(s->master);
  if (s->grad) (void)hipFree(s->grad);
  if (s->vel) (void)hipFree(s->vel);
  if (s->gacc) (void)hipFree(s->gacc);
  for (char* v : s->ver) if (v) (void)hipFree(v);
  if (s->stash) (void)hipFree(s->stash);
  if (s->work) (void)hipFree(s->work);
  delete s;
}

}  // namespace

extern "C" rv_status rv_stage_create(const rv_stage_desc* d, rv_stage** out) {
  if (!d || !out) return RV_E_INVAL;
  *out = nullptr;
  if (d->kind != RV_MLP && d->kind != RV_DECODER) return RV_E_INVAL;
  if (d->n_layers < 1 || d->n_layers > 1024 || !d->dims || d->microbatch < 1 || d->tau < 0 ||
      d->tau > 1024)
    return RV_E_INVAL;
  if (!(d->eta == d->eta)) return RV_E_INVAL;
  if (d->kind == RV_MLP && d->dtype != RV_F32) return RV_E_INVAL;
  if (d->kind == RV_DECODER && d->dtype != RV_BF16) return RV_E_INVAL;
  rv_stage* s = new (std::nothrow) rv_stage();
  if (!s) return RV_E_NOMEM;
  s->kind = d->kind; s->dtype = d->dtype; s->n_layers = d->n_layers;
  s->microbatch = d->microbatch; s->tau = d->tau; s->eta = d->eta;
  s->ln_eps = d->ln_eps > 0.f ? d->ln_eps : 1e-5f;
  s->st = (hipStream_t)d->stream;
  int nd = d->kind == RV_MLP ? d->n_layers + 1 : 4;
  s->dims.assign(d->dims, d->dims + nd);
  rv_status rc = d->kind == RV_MLP ? rv_mlp_plan(s) : rv_dec_plan(s);
  if (rc != RV_OK) { free_all(s); return rc; }
  s->ver_elem = s->dtype == RV_BF16 ? 2 : 4;
  const int ns = s->tau + 1;        // stash slots
  const int nv = s->tau + 2;        // weight versions
  s->ver.assign(nv, nullptr);
  s->ver_ref.assign(nv, 0);
  s->slots.assign(ns, rv_slot());
  bool ok = hipMalloc((void**)&s->master, s->P * 4) == hipSuccess &&
            hipMalloc((void**)&s->grad, s->P * 4) == hipSuccess;
  for (int i = 0; ok && i < nv; ++i) ok = hipMalloc((void**)&s->ver[i], s->P * s->ver_elem) == hipSuccess;
  if (ok && s->slot_bytes) ok = hipMalloc((void**)&s->stash, s->slot_bytes * ns) == hipSuccess;
  if (ok && s->work_bytes) ok = hipMalloc((void**)&s->work, s->work_bytes) == hipSuccess;
  if (!ok) { (void)hipGetLastError(); free_all(s); return RV_E_NOMEM; }
  for (int i = 0; i < ns; ++i) s->slots[i].base = s->stash + (size_t)i * s->slot_bytes;
  if (hipMemsetAsync(s->master, 0, s->P * 4, s->st) != hipSuccess ||
      hipMemsetAsync(s->grad, 0, s->P * 4, s->st) != hipSuccess ||
      hipMemsetAsync(s->ver[0], 0, s->P * s->ver_elem, s->st) != hipSuccess) {
    free_all(s); return RV_E_DEVICE;
  }
  if (hipStreamCreateWithFlags(&s->aux, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_join, hipEventDisableTiming) != hipSuccess ||
      hipStreamCreateWithFlags(&s->wgs, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_wg_ready, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_wg_done[0], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_wg_done[1], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_sync_ready, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s->ev_sync_done, hipEventDisableTiming) != hipSuccess) {
    free_all(s); return RV_E_DEVICE;
  }
  s->cur = 0;
  *out = s;
  return RV_OK;
}

extern "C" rv_status rv_stage_destroy(rv_stage* s) {
  if (!s) return RV_E_INVAL;
  (void)hipStreamSynchronize(s->st);
  if (s->aux) (void)hipStreamSynchronize(s->aux);
  if (s->wgs) (void)hipStreamSynchronize(s->wgs);
  free_all(s);
  return RV_OK;
}

extern "C" size_t rv_stage_num_params(const rv_stage* s) { return s ? s->P : 0; }

extern "C" int rv_stage_in_flight(const rv_stage* s) {
  if (!s) return 0;
  int n = 0;
  for (const rv_slot& sl : s->slots) n += sl.live ? 1 : 0;
  return n;
}

extern "C" rv_status rv_stage_set_params(rv_stage* s, const float* flat, size_t n) {
  if (!s || !flat || n != s->P || s->sync_dst >= 0) return RV_E_INVAL;
  if (rv_stage_in_flight(s) != 0) return RV_E_INVAL;
  RV_HIP_TRY(hipMemcpyAsync(s->master, flat, n * 4, hipMemcpyDeviceToDevice, s->st));
  return rv_launch_publish(s->master, s->P, s->ver[s->cur], copy_kind(s), s->st);
}

extern "C" rv_status rv_stage_set_optimizer(rv_stage* s, float momentum, float weight_decay) {
  if (!s || !(momentum >= 0.f) || !(weight_decay >= 0.f) || s->sync_dst >= 0) return RV_E_INVAL;
  if (rv_stage_in_flight(s) != 0) return RV_E_INVAL;
  if (!s->vel) {
    if (hipMalloc((void**)&s->vel, s->P * 4) != hipSuccess) { (void)hipGetLastError(); s->vel = nullptr; return RV_E_NOMEM; }
  }
  RV_HIP_TRY(hipMemsetAsync(s->vel, 0, s->P * 4, s->st));
  s->momentum = momentum; s->weight_decay = weight_decay;
  return RV_OK;
}

extern "C" rv_status rv_stage_set_accumulation(rv_stage* s, int microbatches) {
  if (!s || microbatches < 1) return RV_E_INVAL;
  if (rv_stage_in_flight(s) != 0) return RV_E_INVAL;
  if (microbatches > 1 && !s->gacc) {
    if (hipMalloc((void**)&s->gacc, s->P * 4) != hipSuccess) { (void)hipGetLastError(); s->gacc = nullptr; return RV_E_NOMEM; }
  }
  s->accum = microbatches;
  s->acc_count = 0;     // a group in progress is dropped
  return RV_OK;
}

extern "C" rv_status rv_stage_defer_update(rv_stage* s, int on) {
  if (!s) return RV_E_INVAL;
  if (on && (s->accum > 1 || s->vel)) return RV_E_INVAL;   // the folded step is the plain one of Alg. 2
  s->defer = on != 0;
  return RV_OK;
}

extern "C" rv_status rv_cluster_sync_fork(rv_stage* const* stages, int C, int R, int pending, int flags,
                                          void* sync_stream) {
  if (!stages || C < 1 || C > 64 || R < 1 || pending < -1 || pending >= C || (flags & ~1)) return RV_E_INVAL;
  const bool state = (flags & 1) != 0;
  if (state && pending >= 0) return RV_E_INVAL;   // the folded step is the plain one of Alg. 2
  float* masters[64];
  float* vels[64];
  for (int c = 0; c < C; ++c) {
    rv_stage* s = stages[c];
    if (!s || s->P != stages[0]->P || s->dtype != stages[0]->dtype || s->st != stages[0]->st) return RV_E_INVAL;
    for (int k = 0; k < c; ++k) if (stages[k] == s) return RV_E_INVAL;
    if (s->accum > 1 && s->acc_count != 0) return RV_E_INVAL;   // a gradient group is open
    if (s->sync_dst >= 0) return RV_E_INVAL;                    // an averaging is already under way
    if (state && !s->vel) return RV_E_INVAL;
    masters[c] = s->master;
    vels[c] = s->vel;
  }
  // Every stage needs a version slot that no in-flight microbatch is bound to - and not the
  // current one, which forwards issued before the join still bind to.  With tau+2 slots one
  // exists unless tau+1 microbatches are in flight; then no forward can be admitted before the
  // join (its stash is full) and the current slot, if unreferenced, may be overwritten.
  int dst[64];
  for (int c = 0; c < C; ++c) {
    rv_stage* s = stages[c];
    dst[c] = -1;
    for (size_t v = 0; dst[c] < 0 && v < s->ver.size(); ++v)
      if (s->ver_ref[v] == 0 && (int)v != s->cur) dst[c] = (int)v;
    if (dst[c] < 0 && s->ver_ref[s->cur] == 0 && rv_stage_in_flight(s) > s->tau) dst[c] = s->cur;
    if (dst[c] < 0) return RV_E_STASH_FULL;
  }
  const rv_stage* p = pending >= 0 ? stages[pending] : nullptr;
  if (p && !p->grad_valid) return RV_E_INVAL;   // no deferred gradient to fold in
  rv_stage* owner = stages[0];
  hipStream_t st = owner->st, ss = (hipStream_t)sync_stream;
  const bool forked = ss != st;
  if (forked) {   // the averaging follows everything enqueued on the stages' stream so far
    RV_HIP_TRY(hipEventRecord(owner->ev_sync_ready, st));
    RV_HIP_TRY(hipStreamWaitEvent(ss, owner->ev_sync_ready, 0));
  }
  RV_TRY(rv_cluster_average(masters, C, owner->P, R, nullptr, 1, p ? p->grad : nullptr, pending >= 0 ? pending : 0,
                            p ? p->eta : 0.f, ss));
  if (state) RV_TRY(rv_cluster_average(vels, C, owner->P, R, nullptr, 1, nullptr, 0, 0.f, ss));
  for (int c = 0; c < C; ++c) {
    rv_stage* s = stages[c];
    RV_TRY(rv_launch_publish(s->master, s->P, s->ver[dst[c]], copy_kind(s), ss));
  }
  if (forked) RV_HIP_TRY(hipEventRecord(owner->ev_sync_done, ss));
  for (int c = 0; c < C; ++c) {
    stages[c]->sync_dst = dst[c];
    stages[c]->sync_owner = forked ? owner : nullptr;
  }
  return RV_OK;
}

extern "C" rv_status rv_cluster_sync_join(rv_stage* const* stages, int C) {
  if (!stages || C < 1 || C > 64) return RV_E_INVAL;
  for (int c = 0; c < C; ++c)
    if (!stages[c] || stages[c]->sync_dst < 0) return RV_E_INVAL;
  for (int c = 0; c < C; ++c) {
    rv_stage* s = stages[c];
    if (s->sync_owner) RV_HIP_TRY(hipStreamWaitEvent(s->st, s->sync_owner->ev_sync_done, 0));
    s->cur = s->sync_dst;      // the mean is the newest weight version from here on
    s->sync_dst = -1;
    s->sync_owner = nullptr;
  }
  return RV_OK;
}

extern "C" rv_status rv_cluster_sync(rv_stage* const* stages, int C, int R, int pending) {
  if (!stages || C < 1 || !stages[0]) return RV_E_INVAL;
  RV_TRY(rv_cluster_sync_fork(stages, C, R, pending, 0, stages[0]->st));
  return rv_cluster_sync_join(stages, C);
}

extern "C" rv_status rv_stage_profile(rv_stage* s, int on) {
  if (!s) return RV_E_INVAL;
  s->prof_on = on != 0;
  return RV_OK;
}

extern "C" rv_status rv_stage_profile_read(rv_stage* s, int* launches, float* mean_us) {
  if (!s || !launches || !mean_us) return RV_E_INVAL;
  RV_HIP_TRY(hipStreamSynchronize(s->st));
  if (s->aux) RV_HIP_TRY(hipStreamSynchronize(s->aux));
  if (s->wgs) RV_HIP_TRY(hipStreamSynchronize(s->wgs));
  double sum_ms = 0.0;
  int n = 0;
  rv_status rc = RV_OK;
  for (size_t i = 0; i + 1 < s->prof_ev.size(); i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, s->prof_ev[i], s->prof_ev[i + 1]) == hipSuccess) { sum_ms += ms; ++n; }
    else { (void)hipGetLastError(); rc = RV_E_DEVICE; }
  }
  for (hipEvent_t ev : s->prof_ev) if (ev) (void)hipEventDestroy(ev);
  s->prof_ev.clear();
  *launches = n;
  *mean_us = n ? (float)(sum_ms * 1e3 / n) : 0.f;
  return rc;
}

extern "C" rv_status rv_stage_get_params(const rv_stage* s, float* flat_out, size_t n) {
  if (!s || !flat_out || n != s->P || s->sync_dst >= 0) return RV_E_INVAL;
  RV_HIP_TRY(hipMemcpyAsync(flat_out, s->master, n * 4, hipMemcpyDeviceToDevice, s->st));
  return RV_OK;
}

extern "C" rv_status rv_stage_keep_grad(rv_stage* s, int on) {
  if (!s) return RV_E_INVAL;
  s->keep_grad = on != 0;
  return RV_OK;
}

extern "C" rv_status rv_stage_last_grad(const rv_stage* s, float* flat_out, size_t n) {
  if (!s || !flat_out || n != s->P) return RV_E_INVAL;
  if (!s->grad_valid) return RV_E_INVAL;   // no backward yet, or its gradient was consumed where it was produced
  RV_HIP_TRY(hipMemcpyAsync(flat_out, s->grad, n * 4, hipMemcpyDeviceToDevice, s->st));
  return RV_OK;
}

// delayed update (Eq. 2, or its momentum / weight-decay variant) of parameters [off, off+n)
// into the version slot chosen for this backward
rv_status rv_stage_update_range(rv_stage* s, size_t off, size_t n, hipStream_t st) {
  const int kind = s->dtype == RV_BF16 ? 1 : 2;
  const float* g = s->grad + off;
  if (s->defer) return RV_OK;   // the update stays pending
  if (s->accum > 1) {   // sum the group's gradients; only its last microbatch updates
    RV_TRY(rv_launch_accumulate(s->gacc + off, g, n, s->acc_count == 0, st));
    if (s->acc_count + 1 < s->accum) return RV_OK;
    g = s->gacc + off;
  }
  void* copy = (char*)s->ver[s->upd_dst] + off * s->ver_elem;
  if (s->vel)
    return rv_launch_update_momentum(s->master + off, g, s->vel + off, n, s->eta, s->momentum, s->weight_decay,
                                     copy, kind, st);
  return rv_launch_update(s->master + off, g, n, s->eta, copy, kind, st);
}

namespace {

// forward branch: bind to a free slot and the newest version, enqueue on s->st
rv_status do_forward(rv_stage* s, int64_t mb_id, const void* in, void* out) {
  int free_i = -1;
  for (size_t i = 0; i < s->slots.size(); ++i)
    if (!s->slots[i].live) { free_i = (int)i; break; }
  if (free_i < 0) return RV_E_STASH_FULL;
  rv_slot& sl = s->slots[free_i];
  sl.ver = s->cur;
  rv_status rc = s->kind == RV_MLP ? rv_mlp_forward(s, sl, in, out) : rv_dec_forward(s, sl, in, out);
  if (rc != RV_OK) { sl.ver = -1; return rc; }
  sl.live = true; sl.mb = mb_id;
  s->ver_ref[s->cur] += 1;
  return RV_OK;
}

// backward branch + update, enqueued on s->st
rv_status do_backward(rv_stage* s, int slot_i, const void* grad_out, void* grad_in) {
  rv_slot& sl = s->slots[slot_i];
  // The updated block is published as a new version in a slot that no in-flight microbatch is
  // bound to - not even this one, whose version the backward is still reading while the first
  // pieces of the new one are written (tau+2 slots, at most tau+1 of them referenced).  The slot
  // is chosen before the backward so that a stage kind may update layer by layer as the
  // gradients complete.  With gradient accumulation only the last microbatch of a group
  // updates; the others leave the current version in force.
  const bool updates = !s->defer && s->acc_count + 1 >= s->accum;
  int dst = -1;
  if (updates) {
    for (size_t v = 0; dst < 0 && v < s->ver.size(); ++v)
      if (s->ver_ref[v] == 0) dst = (int)v;
    if (dst < 0) return RV_E_DEVICE;  // unreachable by the counting argument above
  }
  // Plain Eq. 2 on a decoder stage is applied in the epilogues that produce the gradient (the
  // weight-gradient products, the column reductions); momentum, accumulation and deferred steps
  // take the separate update kernels.
  s->fused = s->kind == RV_DECODER && updates && s->accum == 1 && !s->vel;
  s->upd_dst = dst;
  rv_status rc;
  if (s->kind == RV_MLP) {
    rc = rv_mlp_backward(s, sl, grad_out, grad_in);
    if (rc == RV_OK) rc = rv_stage_update_range(s, 0, s->P, s->st);
  } else {
    rc = rv_dec_backward(s, sl, grad_out, grad_in);   // updates block by block
  }
  if (rc != RV_OK) return rc;   // (a failed launch leaves the stage unusable)
  s->grad_valid = !s->fused || s->keep_grad;
  sl.live = false;
  s->ver_ref[sl.ver] -= 1;
  sl.ver = -1;
  if (updates) { s->cur = dst; s->acc_count = 0; }
  else if (!s->defer) s->acc_count += 1;
  return RV_OK;
}

}  // namespace

extern "C" rv_status rv_stage_forward(rv_stage* s, int64_t mb_id, const void* in, void* out) {
  if (!s || !in || !out) return RV_E_INVAL;
  if (find_slot(s, mb_id) >= 0) return RV_E_DUP_MB;
  return do_forward(s, mb_id, in, out);
}

extern "C" rv_status rv_stage_backward(rv_stage* s, int64_t mb_id, const void* grad_out, void* grad_in) {
  if (!s || !grad_out) return RV_E_INVAL;
  if (s->sync_dst >= 0) return RV_E_INVAL;   // the parameters are being averaged on another stream
  int i = find_slot(s, mb_id);
  if (i < 0) return RV_E_UNKNOWN_MB;
  return do_backward(s, i, grad_out, grad_in);
}

extern "C" rv_status rv_stage_step(rv_stage* s, int64_t fwd_mb, const void* in, void* out, int64_t bwd_mb,
                                   const void* grad_out, void* grad_in) {
  if (!s || !in || !out || !grad_out || s->sync_dst >= 0) return RV_E_INVAL;
  if (find_slot(s, fwd_mb) >= 0) return RV_E_DUP_MB;
  if (fwd_mb == bwd_mb) {  // tau = 0: the backward needs this very forward; nothing to overlap
    RV_TRY(do_forward(s, fwd_mb, in, out));
    return do_backward(s, find_slot(s, bwd_mb), grad_out, grad_in);
  }
  const int bi = find_slot(s, bwd_mb);
  if (bi < 0) return RV_E_UNKNOWN_MB;
  if (rv_stage_in_flight(s) > s->tau) return RV_E_STASH_FULL;   // no free slot for the forward
  // fork: the backward of the old microbatch runs on the auxiliary stream beside the
  // forward of the new one; both see the weights as they are before this step's update.
  hipStream_t main_st = s->st;
  RV_HIP_TRY(hipEventRecord(s->ev_fork, main_st));
  RV_HIP_TRY(hipStreamWaitEvent(s->aux, s->ev_fork, 0));
  s->in_step = true;
  rv_status rc = do_forward(s, fwd_mb, in, out);
  if (rc == RV_OK) {
    s->st = s->aux;
    rc = do_backward(s, bi, grad_out, grad_in);
    s->st = main_st;
  }
  s->in_step = false;
  // join even after a failure so the caller's stream stays ordered behind the aux work
  hipError_t e1 = hipEventRecord(s->ev_join, s->aux);
  hipError_t e2 = hipStreamWaitEvent(main_st, s->ev_join, 0);
  if (rc != RV_OK) return rc;
  return (e1 == hipSuccess && e2 == hipSuccess) ? RV_OK : RV_E_DEVICE;
}

extern "C" const char* rv_strerror(rv_status st) {
  switch (st) {
    case RV_OK: return "ok";
    case RV_E_INVAL: return "invalid argument";
    case RV_E_STASH_FULL: return "tau+1 microbatches already in flight";
    case RV_E_UNKNOWN_MB: return "microbatch id not in flight";
    case RV_E_DUP_MB: return "microbatch id already in flight";
    case RV_E_NOMEM: return "out of memory";
    case RV_E_DEVICE: return "HIP call failed";
  }
  return "unknown status";
}
