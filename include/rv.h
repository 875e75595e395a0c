/*
 * rv.h - C ABI of the stage-step / cluster-average library for one MI355X (gfx950).
 *
 * The calls follow the problem statement of "Ravnest: Decentralized Asynchronous
 * Training on Heterogeneous Devices" (arXiv 2401.01728):
 *
 *   - a peer ("stage") owns one contiguous block x_{c,p} of the model (Eq. 1),
 *   - it runs forward passes on arriving activations and, on arriving gradients,
 *     a backward pass followed at once by the stale-gradient update of Eq. 2
 *     (Alg. 1, the two branches of the peer loop),
 *   - clusters average their parameters with a Parallel Multi-Ring All-Reduce
 *     (section 3.2); here all C replicas live in one GPU's memory and only the
 *     arithmetic of that reduction is performed.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary process memory.  The library never takes ownership
 *     of a caller buffer.
 *   - Every call validates its arguments on the host, enqueues its work on the
 *     stage's (or the given) hipStream_t and returns without synchronising.
 *     A caller buffer may be reused once the stream has passed the call.
 *   - Errors are returned, never thrown.  Arguments and stage state are checked before
 *     anything is enqueued: after RV_E_INVAL, RV_E_STASH_FULL, RV_E_UNKNOWN_MB, RV_E_DUP_MB
 *     or RV_E_NOMEM the stage state is unchanged.  RV_E_DEVICE means a HIP call failed,
 *     possibly with part of the call's work already enqueued: the stage (for
 *     rv_cluster_sync: every stage passed) is then fit only for rv_stage_destroy.
 *
 * Canonical flat parameter order (what set/get_params, last_grad and the
 * average see), layers in forward order, every matrix row-major [in, out]:
 *   MLP stage      : W_0, b_0, W_1, b_1, ...
 *   decoder block  : ln1.gamma[d], ln1.beta[d], Wqkv[d,3d] (column thirds q|k|v,
 *                    heads contiguous inside a third), bqkv[3d], Wo[d,d], bo[d],
 *                    ln2.gamma[d], ln2.beta[d], W1[d,f], b1[f], W2[f,d], b2[d]
 */
#ifndef RV_H
#define RV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rv_stage rv_stage; /* opaque, library-owned */

typedef enum {
  RV_OK = 0,
  RV_E_INVAL = -1,      /* bad argument (null pointer, non-positive size, d % heads != 0, ...) */
  RV_E_STASH_FULL = -2, /* forward with tau+1 microbatches already in flight            */
  RV_E_UNKNOWN_MB = -3, /* backward of a microbatch id that is not in flight             */
  RV_E_DUP_MB = -4,     /* forward of a microbatch id that is already in flight          */
  RV_E_NOMEM = -5,      /* device or host allocation failed                              */
  RV_E_DEVICE = -6      /* a HIP call failed                                             */
} rv_status;

typedef enum { RV_MLP = 0, RV_DECODER = 1 } rv_kind;
typedef enum { RV_F32 = 0, RV_BF16 = 1 } rv_dtype;

/*
 * Description of one stage.
 *   kind RV_MLP     : n_layers Linear layers with ReLU between them (none after
 *                     the last); dims = n_layers+1 widths; dtype must be RV_F32;
 *                     activations are fp32 [microbatch, width].
 *   kind RV_DECODER : n_layers pre-LayerNorm decoder blocks (causal self
 *                     attention, GELU feed-forward); dims = {d_model, n_heads,
 *                     d_ffn, seq}; dtype must be RV_BF16: activations and
 *                     gradients at the boundary are bf16 [microbatch, seq, d_model],
 *                     matrix products take bf16 operands with fp32 accumulation,
 *                     the master parameters are fp32.  d_model / n_heads must be
 *                     64 or 128; d_model, d_ffn multiples of 64; seq a multiple of 64.
 *   tau             : largest number of updates that may happen between a
 *                     microbatch's forward and its backward (the staleness bound
 *                     of Eq. 2); the stage keeps tau+1 activation-stash slots and
 *                     tau+2 weight versions (tau+1 in use by microbatches in flight, one
 *                     being written by the update).
 *   eta             : learning rate of Eq. 2.
 *   stream          : hipStream_t (borrowed); NULL = the default stream.
 */
typedef struct {
  int32_t kind;
  int32_t dtype;
  int32_t n_layers;
  const int64_t* dims; /* host */
  int32_t microbatch;
  int32_t tau;
  float eta;
  float ln_eps;
  void* stream;
} rv_stage_desc;

/* Allocates master parameters (zero), gradient buffer, tau+2 weight versions and
 * tau+1 stash slots on the current device.  RV_E_INVAL / RV_E_NOMEM / RV_E_DEVICE. */
rv_status rv_stage_create(const rv_stage_desc* desc, rv_stage** out);
rv_status rv_stage_destroy(rv_stage* s);

/* Length P of the flat parameter vector (0 for a NULL stage). */
size_t rv_stage_num_params(const rv_stage* s);

/* Number of microbatches forwarded and not yet backwarded. */
int rv_stage_in_flight(const rv_stage* s);

/* Replace the fp32 master vector (device [n], n == P) and make it the current
 * weight version.  Only legal with no microbatch in flight (RV_E_INVAL otherwise). */
rv_status rv_stage_set_params(rv_stage* s, const float* flat, size_t n);
/* Copy the fp32 master vector into flat_out (device [n], n == P). */
rv_status rv_stage_get_params(const rv_stage* s, float* flat_out, size_t n);
/* Copy the parameter gradient computed by the most recent backward (device [n]).  A decoder
 * stage taking the plain step of Eq. 2 applies it inside the kernels that produce the gradient
 * and keeps no copy of it unless rv_stage_keep_grad was switched on: RV_E_INVAL then, and
 * before the first backward. */
rv_status rv_stage_last_grad(const rv_stage* s, float* flat_out, size_t n);
/* on != 0: backward calls also store the parameter gradient (4 more bytes written per
 * parameter), for rv_stage_last_grad.  Off by default.  MLP stages and the momentum /
 * accumulation / deferred-update variants always have it. */
rv_status rv_stage_keep_grad(rv_stage* s, int on);

/*
 * Optional: the optimiser of the paper's single-cluster experiments (section 4.1, SGD
 * with momentum and weight decay) in place of the plain step of Eq. 2:
 *   d = g + weight_decay * w;  v <- momentum * v + d;  w <- w - eta * v
 * Allocates the velocity buffer (fp32 [P]) on first use and zeroes it.  Only legal with no
 * microbatch in flight.  momentum = weight_decay = 0 reproduces Eq. 2 exactly.
 */
rv_status rv_stage_set_optimizer(rv_stage* s, float momentum, float weight_decay);

/*
 * Optional: gradient accumulation as in the paper's multi-cluster experiment (section 4.2): the
 * gradients of `microbatches` consecutive backward calls are summed and the update (Eq. 2, or
 * the optimiser set above) is applied once, with the sum, by the last of them; the others
 * leave the parameters and the current weight version as they are.  1 = update on every
 * backward (the default).  Only legal with no microbatch in flight; a group in progress is
 * dropped.  Allocates an fp32 [P] accumulator on first use.  rv_stage_last_grad keeps
 * returning the last microbatch's own gradient.
 */
rv_status rv_stage_set_accumulation(rv_stage* s, int microbatches);

/*
 * Forward branch of Alg. 1: out = forward_pass(x_{c,p}, in) at the CURRENT
 * parameters.  Binds mb_id to a stash slot and to the current weight version.
 * in/out: device, MLP fp32 [microbatch, dims[0]] -> [microbatch, dims[n_layers]];
 * decoder bf16 [microbatch, seq, d_model] -> same shape.
 * RV_E_STASH_FULL when tau+1 microbatches are in flight; RV_E_DUP_MB.
 */
rv_status rv_stage_forward(rv_stage* s, int64_t mb_id, const void* in, void* out);

/*
 * Backward branch of Alg. 1 with the update of Eq. 2: computes the exact
 * gradient of the block at the weights and activations of mb_id's forward
 * (the stale gradient g^{k - tau_k}), writes the gradient for the preceding
 * peer to grad_in (may be NULL), applies x <- x - eta * g to this stage's
 * block only (Eq. 4) and publishes the result as the newest weight version.
 * Any in-flight id is legal.  RV_E_UNKNOWN_MB.
 */
rv_status rv_stage_backward(rv_stage* s, int64_t mb_id, const void* grad_out, void* grad_in);

/*
 * One steady-state stage step: rv_stage_forward(fwd_mb, in, out) and
 * rv_stage_backward(bwd_mb, grad_out, grad_in) issued together, with the same result as
 * calling them in that order: the forward runs at the parameters in force BEFORE this
 * step's update (it does not wait for the gradient of bwd_mb - the zero-bubble property
 * of section 3.1), the backward at the version stashed for bwd_mb, then the update of
 * Eq. 2.  The two halves are independent and are enqueued on separate streams (the forward on
 * the stage's stream; the backward's chain dy -> dx on an internal one; its parameter-gradient
 * work - weight-gradient products, bias and LayerNorm reductions, the block-by-block update -
 * on a third; forked and joined with events, default priorities), so their kernels overlap on
 * the GPU; all work is ordered after what was on the stage's stream at the call and before
 * what is enqueued on it afterwards.  With fwd_mb == bwd_mb (tau = 0) the halves run in
 * sequence.  Errors as for the two calls; RV_E_STASH_FULL if no slot is free for fwd_mb.
 */
rv_status rv_stage_step(rv_stage* s, int64_t fwd_mb, const void* in, void* out, int64_t bwd_mb,
                        const void* grad_out, void* grad_in);

/*
 * The update of Eq. 2 on a bare vector: w[i] <- w[i] - eta * g[i] (one fused
 * multiply-add in fp32), optionally also emitting the bf16 rounding of the new
 * w into bf16_out (device [n] of 16-bit words, may be NULL).  All device.
 */
rv_status rv_block_update(float* w, const float* g, size_t n, float eta, void* bf16_out,
                          void* stream);

/*
 * The all-reduce branch of the method's outer loop (Alg. 2): C clusters hold one stage each for
 * the same block of layers (same parameter count and dtype, created on the same stream, all
 * resident in this GPU's HBM).  rv_cluster_sync replaces every stage's parameters by their
 * ring-partitioned mean over R rings (rv_cluster_average with write-back on the fp32 master
 * vectors) and makes the mean each stage's current weight version; microbatches in flight keep
 * the versions they were forwarded with.  pending = index of the stage whose last backward ran
 * with its update deferred: its step x - eta * g is folded into the mean (Eq. 17); -1 = none.
 * RV_E_STASH_FULL if a stage has no version slot free of in-flight microbatches.
 *
 * rv_stage_defer_update(s, 1): following backward / step calls compute grad_in and the
 * parameter gradient but leave parameters and weight version untouched (Alg. 2 folds the
 * sampled peer's step into the all-reduce at an averaging step); 0 restores Eq. 2 on every
 * backward.  Not combinable with gradient accumulation or the momentum optimiser.
 */
rv_status rv_stage_defer_update(rv_stage* s, int on);
rv_status rv_cluster_sync(rv_stage* const* stages, int C, int R, int pending);

/*
 * The same all-reduce started on ANOTHER stream, so that the stages' own stream keeps working
 * beside it (the clusters of the paper do not stop while their parameters are averaged):
 * rv_cluster_sync_fork orders the averaging behind everything enqueued on the stages' stream so
 * far and enqueues it on sync_stream (hipStream_t; the stages' own stream is allowed and gives
 * rv_cluster_sync); the mean is written into version slots no microbatch is bound to.  Until
 * rv_cluster_sync_join, forwards are legal on every stage and run at the version in force before
 * the averaging (one more update of staleness for those microbatches, exactly as if they had been
 * forwarded just before it); backward / step / set_params / get_params / set_optimizer return
 * RV_E_INVAL.  rv_cluster_sync_join makes the stages' stream wait for the averaging and the mean
 * the current weight version.  A cluster that is a chain of peers is averaged by one fork / join
 * pair per peer position.
 * flags bit 0: also average the optimiser state (the momentum buffers of rv_stage_set_optimizer,
 * required on every stage then) in the same cycle; not combinable with a pending step.
 */
rv_status rv_cluster_sync_fork(rv_stage* const* stages, int C, int R, int pending, int flags,
                               void* sync_stream);
rv_status rv_cluster_sync_join(rv_stage* const* stages, int C);

/* The momentum / weight-decay step above on bare vectors; v (device [n]) is read and updated. */
rv_status rv_block_update_momentum(float* w, const float* g, float* v, size_t n, float eta, float momentum,
                                   float weight_decay, void* bf16_out, void* stream);

/*
 * Arithmetic of one cycle of Parallel Multi-Ring All-Reduce (section 3.2) over C
 * replicas of an n-vector that all reside on this GPU.
 *   replicas     host array of C device pointers, each fp32 [n]; must not alias
 *                one another or mean_out.  1 <= C <= 64.
 *   R            number of rings, 1 <= R <= 4096.  Ring r owns elements
 *                [floor(r n / R), floor((r+1) n / R)); inside it chunk j owns
 *                [lo + floor(j S / C), lo + floor((j+1) S / C)), S the segment size.
 *                Chunk j is summed in ring order x_j + x_{j+1} + ... + x_{j-1}
 *                (indices mod C, fp32, left to right) and divided by C once.
 *   mean_out     device [n] or NULL (NULL only with write_back).
 *   write_back   nonzero: every replica is overwritten with the mean, the state
 *                the paper's cycle ends in.
 *   grad,grad_replica,eta   if grad != NULL (device [n]) replica grad_replica
 *                enters the average as x - eta*grad (Alg. 2, the all-reduce
 *                branch), so the mean moves by -(eta/C) grad (Eq. 17).  The
 *                product and the subtraction are rounded separately.
 * RV_E_INVAL on bad arguments.  Pointers that are not 16-byte aligned are
 * accepted (slower path).
 */
rv_status rv_cluster_average(float* const* replicas, int C, size_t n, int R, float* mean_out,
                             int write_back, const float* grad, int grad_replica, float eta,
                             void* stream);

/*
 * The same cycle with rings of UNEQUAL size (section 3.2: clusters split the model
 * differently, a ring covers the parameters two neighbouring peers share, so segment sizes
 * differ and a peer may sit in several rings).  ring_offsets: host array of R+1 element
 * offsets, ring_offsets[0] = 0 <= ... <= ring_offsets[R] = n (empty rings allowed),
 * 1 <= R <= 64.  Ring r owns [ring_offsets[r], ring_offsets[r+1]); chunks, summation order
 * and every other argument as in rv_cluster_average.  RV_E_INVAL on a malformed table.
 */
rv_status rv_cluster_average_v(float* const* replicas, int C, size_t n, const int64_t* ring_offsets,
                               int R, float* mean_out, int write_back, const float* grad,
                               int grad_replica, float eta, void* stream);

/*
 * Measurement aid (no part of the method): while on, a decoder stage brackets every launch of
 * the kernel that dominates its step - the grouped weight-gradient product, which computes
 * dW2 | dW1 | dWo | dWqkv of one block in one to three launches - with HIP events on the stream
 * that launch goes to, inside whatever else the step has running.  rv_stage_profile_read waits for the stage's streams, returns the number
 * of launches bracketed since the last read and their mean duration in microseconds, and
 * forgets them.  Events are created per launch: keep it off outside measurements.
 */
rv_status rv_stage_profile(rv_stage* s, int on);
rv_status rv_stage_profile_read(rv_stage* s, int* launches, float* mean_us);

const char* rv_strerror(rv_status st);

#ifdef __cplusplus
}
#endif
#endif /* RV_H */
