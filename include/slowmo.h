/*
 * slowmo.h -- C ABI of the Slow Momentum optimizer hot path for one AMD
 * MI355X (gfx950).
 *
 * The library runs, for m logical workers whose parameter replicas all live
 * on one GPU, the per-element work of Algorithm 1 ("Slow Momentum"):
 * tau base-optimizer steps per worker (directions of Table C.1, Appendix C:
 * SGD with Nesterov momentum, or Adam), then the outer step (exact average,
 * slow-momentum update Eq. (2), outer-iterate update Eq. (3)) and the copy of
 * the new iterate into every replica.
 *
 * Conventions
 *  - All pointers named "device" are HIP device pointers; everything else is
 *    host memory that may be freed as soon as the call returns.
 *  - Parameters are fp32.  Gradients are fp32 or bf16 (widened exactly).
 *    State (x0, u, h, v) is fp32.  All arithmetic is fp32.
 *  - Tensor lists are worker-major: entry [i * n_tensors + j] belongs to
 *    worker i, tensor j.  Tensor j has numel[j] contiguous elements on every
 *    worker.  Pointers need element alignment only (4 bytes fp32, 2 bytes
 *    bf16); 16-byte alignment selects the vectorized path.
 *  - Ownership: parameters, gradients and the state workspace belong to the
 *    caller.  The library keeps the parameter pointers and the workspace for
 *    the context's lifetime and never frees them; they must not overlap.
 *  - Streams: work is enqueued on the hipStream_t passed as `stream` (NULL =
 *    the default stream) and the step calls return without synchronizing
 *    (create, set_tensor_hparams, export and import do wait; they say so).  All
 *    calls on one context must be issued on one stream or be ordered by the
 *    caller.  A context is not thread-safe.
 *  - Gradient pointers: the library keeps the 16 most recently used distinct
 *    pointer tables on the device; a call whose `grads` array equals one of them
 *    uploads nothing.
 *  - Graph capture: in that case slowmo_local_step, slowmo_outer_step and
 *    slowmo_local_outer_step only launch kernels (no copies, no synchronization,
 *    no memset) and may be recorded into a HIP graph (pass every gradient set
 *    once before capturing, and no more than 16 distinct ones while the graph
 *    is in use).  Kernel arguments are fixed at capture time: the learning
 *    rates, the first/last-step handling of the RESET policy and Adam's bias
 *    corrections.  A captured outer iteration of the SGD base therefore replays
 *    correctly any number of times; one of the Adam base does not (its bias
 *    correction changes every step).  The context's counters advance when the
 *    calls are recorded, not when the graph is replayed.  slowmo_mix_step,
 *    slowmo_local_mix_step and slowmo_debias upload a small table with every
 *    call (from a staging buffer that later calls reuse) and keep the push-sum
 *    weights on the host: do not record them into a graph.
 *  - Errors: every entry point returns a slowmo_status; nothing aborts or
 *    throws.  Arguments, call order and alignment are checked, and every table
 *    a call needs is planned and on its way to the device, before the call's
 *    first kernel is launched; counters and push-sum weights advance after its
 *    last launch was accepted.  A call that fails therefore leaves the
 *    context's state unchanged, with one exception: some calls issue several
 *    kernels or copies (slowmo_mix_step and slowmo_local_mix_step launch one
 *    kernel per connected group of workers; slowmo_local_outer_step and
 *    slowmo_local_mix_step launch two kernels when a pointer is not 16-byte
 *    aligned; slowmo_outer_step and slowmo_local_outer_step launch one kernel
 *    for the whole 65 536-element pieces of the tensors and one for the rest
 *    when the tensor list has at least 160 such pieces -- the former from 16
 *    workers on, the latter from 8 on under SLOWMO_BUF_RESET;
 *    slowmo_import_state copies up to four arrays).  If the HIP
 *    runtime refuses one of them after an earlier one was issued, device
 *    memory is partly updated and cannot be rolled back: the call returns
 *    SLOWMO_ERR_HIP with a message that says so, counters and weights keep
 *    their old values, and every later step call on that context returns
 *    SLOWMO_ERR_STATE.  Destroy such a context.
 *    slowmo_last_error() gives a message for the most recent failure.
 */
#ifndef SLOWMO_H
#define SLOWMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct slowmo_ctx slowmo_ctx; /* opaque */

typedef enum {
  SLOWMO_OK = 0,
  SLOWMO_ERR_ARG = -1,   /* null pointer, size or hyper-parameter out of range, bad enum */
  SLOWMO_ERR_STATE = -2, /* call out of sequence (see local/outer step) */
  SLOWMO_ERR_ALIGN = -3, /* pointer not aligned to its element size / workspace not 256-byte aligned */
  SLOWMO_ERR_HIP = -4,   /* a HIP runtime call failed (no device, launch failure, ...) */
  SLOWMO_ERR_NOMEM = -5  /* workspace too small, or host allocation failed */
} slowmo_status;

/* Base optimizer: the rows "SGD" and "Adam" of Table C.1. */
typedef enum { SLOWMO_SGD_NESTEROV = 0, SLOWMO_ADAM = 1 } slowmo_base;

/* What happens to the base optimizer's buffers at the start of an outer
 * iteration (Algorithm 1 line 2; Appendix B.4).  RESET: h (and v, and Adam's
 * step count) restart from zero -- the paper's default for SGD.  MAINTAIN:
 * they carry over -- the paper's default for Adam.  AVERAGE: every worker's
 * h (and v) is replaced by the mean over the workers, summed in worker order
 * (Appendix B.4 strategy 3; with alpha = 1, beta = 0 and the SGD base this is
 * the double-averaging scheme of Algorithm C.4); Adam's step count runs on.
 * The averaging is done by slowmo_outer_step in the same kernel. */
typedef enum { SLOWMO_BUF_RESET = 0, SLOWMO_BUF_MAINTAIN = 1, SLOWMO_BUF_AVERAGE = 2 } slowmo_bufpolicy;

typedef enum { SLOWMO_F32 = 0, SLOWMO_BF16 = 1 } slowmo_dtype; /* gradient element type */

/* Inputs of Algorithm 1 plus the base optimizer's hyper-parameters. */
typedef struct {
  int32_t m;           /* number of workers, 1..SLOWMO_MAX_WORKERS */
  int32_t tau;         /* base-optimizer steps per outer iteration, >= 1 */
  float alpha;         /* slow learning rate, > 0 */
  float beta;          /* slow momentum factor, 0 <= beta < 1 */
  int32_t base;        /* slowmo_base */
  int32_t policy;      /* slowmo_bufpolicy */
  int32_t grad_dtype;  /* slowmo_dtype */
  float momentum;      /* SGD: local Nesterov momentum beta_local, 0 <= . < 1 */
  float weight_decay;  /* coupled L2 term added to the gradient: g + wd * x, >= 0 */
  float beta1, beta2;  /* Adam moment factors, 0 <= . < 1 */
  float eps;           /* Adam epsilon (added after the square root), >= 0 */
  int32_t no_average;  /* 0: Algorithm 1 as printed (exact average, line 6).
                          1: the "SlowMo-noaverage" variant of Section 6: line 6 is
                          skipped, every worker applies lines 7-8 to its own replica
                          and keeps its own x0 and u (the workspace grows by
                          2 (m - 1) d floats); not combinable with SLOWMO_BUF_AVERAGE */
} slowmo_config;

#define SLOWMO_MAX_WORKERS 1024

/* Which internal buffer slowmo_get_buffer() returns. */
typedef enum { SLOWMO_BUF_X0 = 0, SLOWMO_BUF_U = 1, SLOWMO_BUF_H = 2, SLOWMO_BUF_V = 3 } slowmo_buffer;

/*
 * Bytes of device workspace a context needs for this configuration and
 * tensor list: x0 and u (one copy each; one per worker with cfg.no_average),
 * h (and v for Adam) per worker, and the tiling and pointer tables.  Returns 0 if the arguments are invalid.  Host-only.
 */
size_t slowmo_state_bytes(const slowmo_config *cfg, int32_t n_tensors, const int64_t *numel);

/*
 * Algorithm 1, "Input" line.  Creates a context over a fixed tensor list.
 *   params : host array of m * n_tensors DEVICE pointers (worker-major) to
 *            the fp32 replicas; kept for the context's lifetime.
 *   state  : DEVICE workspace, 256-byte aligned, at least
 *            slowmo_state_bytes() long; owned by the caller.
 * Effects, enqueued on `stream`: x_{0,0} is taken from worker 0's replica and
 * copied into x0 and into the replicas of workers 1..m-1 (the paper assumes a
 * common starting point; this enforces it); u_0 = 0; h = v = 0.  Unlike the
 * step calls, create waits for `stream` before it returns (its tables are
 * uploaded from temporary host memory).  All argument checks come before the
 * first use of the device.  Needs a HIP device.  Errors: ARG, ALIGN, NOMEM, HIP.
 */
slowmo_status slowmo_create(slowmo_ctx **out, const slowmo_config *cfg, int32_t n_tensors,
                            const int64_t *numel, float *const *params, void *state,
                            size_t state_bytes, void *stream);

/*
 * Algorithm 1 lines 3-5 for one k: one base-optimizer step on all m workers,
 *   x^{(i)} <- x^{(i)} - lr * d^{(i)},  d per Table C.1 (SGD row: h <- mu h + g~,
 *   d = mu h + g~;  Adam row: bias-corrected h / (sqrt(v) + eps)),
 *   g~ = g + weight_decay * x,  x the replica itself (with gossip between the
 *   steps: the push-sum numerator, not the de-biased x / w -- the two agree
 *   whenever every mixing step so far was a permutation, as in the paper).
 * Adam's bias-correction exponent is the number of Adam steps taken so far
 * under the buffer policy, counting this one.
 *   grads : host array of m * n_tensors DEVICE pointers (worker-major) to the
 *           gradients of this step, of the configured dtype; may change from
 *           call to call.  Read only.
 *   lr    : gamma_t for this step, finite and > 0.
 * Errors: ARG, ALIGN, HIP; STATE if tau steps were already taken since the
 * last outer step.
 */
slowmo_status slowmo_local_step(slowmo_ctx *ctx, const void *const *grads, float lr, void *stream);

/*
 * Algorithm 1 lines 6-8 in one pass over the elements:
 *   xbar = (x^{(0)} + x^{(1)} + ... + x^{(m-1)}) / m      (summed in this order)
 *   u   <- beta * u + (x0 - xbar) / lr                     Eq. (2)
 *   x0  <- x0 - (alpha * lr) * u                           Eq. (3)
 *   x^{(i)} <- x0 for every worker i,
 * (with cfg.no_average: per worker i, xbar := x^{(i)}, u^{(i)}, x0^{(i)} in place
 * of the shared ones, x^{(i)} <- x0^{(i)}; Section 6)
 * and applies the buffer policy for the next outer iteration (line 2): RESET
 * arms a flag (no memory is touched), AVERAGE replaces h^{(i)} (and v^{(i)})
 * by their mean over i in the same pass.
 *   lr : gamma_t, finite and > 0 (Eq. (2) divides by it).
 * Errors: ARG, HIP; STATE unless exactly tau local steps were taken since the
 * previous outer step (or since creation).
 */
slowmo_status slowmo_outer_step(slowmo_ctx *ctx, float lr, void *stream);

/*
 * The last local step of an outer iteration and the outer step as one call:
 * the same results, bit for bit, as
 *     slowmo_local_step(ctx, grads, lr, stream);
 *     slowmo_outer_step(ctx, outer_lr, stream);
 * but when cfg.no_average is 0 and every replica and gradient pointer is
 * 16-byte aligned (8 bytes for bf16 gradients) both run in ONE kernel that
 * keeps the stepped replicas in registers for the average: the replicas are
 * read and written once instead of twice (8 m bytes less traffic per element),
 * and the per-worker buffers of this step are not written under the RESET and
 * AVERAGE policies.  Otherwise the two kernels are launched back to back.
 * Errors: as for the two calls; STATE unless exactly tau-1 local steps were
 * taken since the previous outer step.
 */
slowmo_status slowmo_local_outer_step(slowmo_ctx *ctx, const void *const *grads, float lr,
                                      float outer_lr, void *stream);

/*
 * One mixing (gossip) step of stochastic gradient push among the m logical
 * workers: Algorithm C.1, "send / receive / update model parameters", i.e.
 * X <- X P^T of Appendix C.1, with a column-stochastic P in which every
 * worker has at most one in-neighbour besides itself.
 *   in_peer : host array of m worker indices in 0..m-1; worker i receives from
 *             worker in_peer[i] (in_peer[i] == i: from nobody).  A worker may
 *             send to any number of workers.
 * A sender j splits its mass evenly between itself and its outdeg(j)
 * receivers: p(i,j) = 1 / (1 + outdeg(j)) for j == i and j == in_peer[i], so
 *   x^{(i)} <- p(i,i) x^{(i)} + p(i,in_peer[i]) x^{(in_peer[i])}   (old values on the right)
 * for all i at once, in place, and the push-sum weights w_i, kept on the host,
 * mix the same way.  When in_peer is a permutation (the case the paper runs:
 * one message sent and one received per worker) every weight is 1/2 and P is
 * doubly stochastic: equal w_i stay equal.  The w_i start at 1 and return
 * to 1 at every outer step that averages exactly (cfg.no_average == 0).
 * May be called any number of times between local steps; it changes the
 * replicas and the w_i only.
 * Errors: ARG (NULL, an entry outside 0..m-1), HIP.
 */
slowmo_status slowmo_mix_step(slowmo_ctx *ctx, const int32_t *in_peer, void *stream);

/*
 * A local step and the mixing step that follows it as one call (stochastic
 * gradient push as base optimizer, Algorithm C.1, runs this pair tau times per
 * outer iteration): the same results, bit for bit, as
 *     slowmo_local_step(ctx, grads, lr, stream);
 *     slowmo_mix_step(ctx, in_peer, stream);
 * but when every replica and gradient pointer is 16-byte aligned (8 bytes for
 * bf16 gradients) both run in ONE kernel that keeps the stepped replicas in
 * registers for the mix: the replicas are read and written once instead of
 * twice (8 bytes less traffic per worker and element).  Otherwise the two
 * kernels are launched back to back.
 * Errors: as for the two calls.
 */
slowmo_status slowmo_local_mix_step(slowmo_ctx *ctx, const void *const *grads, float lr,
                                    const int32_t *in_peer, void *stream);

/*
 * Inspection: the order in which slowmo_mix_step updates the replicas in
 * place.  Entry e sets, per element,
 *     x[worker] <- keep * own + take * src       (keep * own with NO_SOURCE)
 * where own and src are the values x[worker] and x[source] had BEFORE the
 * step.  They are read from memory unless a flag says that the kernel still
 * holds them: OWN_HELD / SOURCE_HELD -- the operand is the source operand of
 * the closest earlier entry that has one; SOURCE_IS_FIRST -- the operand is
 * the own operand of the closest earlier entry flagged OPENS_CYCLE.  The
 * kernel has SLOWMO_MIX_SAVED_REGISTERS more registers for operands ("saved"),
 * numbered from 1; three 3-bit fields of `flags` (0 = no) refer to them:
 * SLOWMO_MIX_SAVE(flags) = k -- before this entry's source operand replaces the
 * held one (the source operand of the closest earlier entry that has one), the
 * held operand is copied into saved register k, because a later entry needs it
 * again; SLOWMO_MIX_OWN_SAVED(flags) = k / SLOWMO_MIX_SOURCE_SAVED(flags) = k --
 * the operand is the one in saved register k (as a source it also becomes the
 * held operand again).  A sender with several receivers is thus read once even
 * when other senders come in between (as long as a register is free;
 * otherwise it is read again).  The order
 * is valid if no entry reads from memory a worker that an earlier entry has
 * written.  Idle workers (no sender, no receiver) have no entry.  Entries of
 * one connected group of workers are consecutive and the first of them carries
 * GROUP_START; no HELD / IS_FIRST / SAVED flag refers across a group start, and the
 * library runs the groups as separate kernel launches.
 * Writes at most m entries to `out` (host) and returns their number, or -1
 * for bad arguments.  Host-only.
 */
enum {
  SLOWMO_MIX_OWN_HELD = 1,
  SLOWMO_MIX_SOURCE_HELD = 2,
  SLOWMO_MIX_SOURCE_IS_FIRST = 4,
  SLOWMO_MIX_OPENS_CYCLE = 8,
  SLOWMO_MIX_NO_SOURCE = 16,
  SLOWMO_MIX_GROUP_START = 32
};
#define SLOWMO_MIX_SAVED_REGISTERS 4
#define SLOWMO_MIX_SAVE(flags) (((flags) >> 6) & 7)
#define SLOWMO_MIX_OWN_SAVED(flags) (((flags) >> 9) & 7)
#define SLOWMO_MIX_SOURCE_SAVED(flags) (((flags) >> 12) & 7)
typedef struct slowmo_mix_entry {
  int32_t worker;
  int32_t source;
  float keep;      /* p(worker, worker) */
  float take;      /* p(worker, source) */
  int32_t flags;   /* SLOWMO_MIX_* bits */
  int32_t reserved;
} slowmo_mix_entry;
int32_t slowmo_plan_mix(int32_t m, const int32_t *in_peer, slowmo_mix_entry *out);

/* Copies the m push-sum weights w_i (Algorithm C.1) into the HOST array w.
 * Host-only, no device work.  Errors: ARG. */
slowmo_status slowmo_get_pushsum_weights(const slowmo_ctx *ctx, float *w);

/*
 * The de-biased parameters of Algorithm C.1 (last line): z^{(i)} = x^{(i)} / w_i,
 * the point at which worker i evaluates its next gradient.
 *   z : host array of m * n_tensors DEVICE pointers, laid out like `params` of
 *       slowmo_create; z[i * n_tensors + j] receives numel[j] floats.  4-byte
 *       alignment is enough (16 enables vector stores).  The destinations
 *       must not overlap the replicas, the workspace or each other.
 * Reads the replicas and the current w_i; changes no state.  The pointer array
 * is copied before the call returns.  Asynchronous on `stream`.
 * Errors: ARG (NULL), ALIGN, HIP.
 */
slowmo_status slowmo_debias(slowmo_ctx *ctx, float *const *z, void *stream);

/*
 * slowmo_debias for callers that cannot allocate device memory or spare
 * workspace for it: code recorded into a HIP graph, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results bit for bit.
 * The table its kernel reads (the m * n_tensors destination pointers and the
 * m weights), which slowmo_debias places in the caller's workspace, lives here
 * in a static device array inside the library (528 KiB per GPU, held until the
 * process ends), so the call makes no hipMalloc / hipFree and no other
 * allocating call; it fills a pinned staging buffer that slowmo_create
 * allocated, enqueues one copy and one kernel on `stream`.
 *   Limit: m * n_tensors <= SLOWMO_STATIC_MAX_POINTERS, else NOMEM (use
 *   slowmo_debias).
 *   The array is shared by all contexts on a GPU and keeps the previous
 *   call's table; a call overwrites the part it uses and its kernel reads
 *   nothing beyond that, so no clearing is needed.  Calls on ONE stream are
 *   ordered and safe; calls that overlap on one GPU (different streams or
 *   threads, any contexts) race for the array: order them.
 *   The context's device must be the current device.
 * Errors: as slowmo_debias; NOMEM beyond the limit; STATE if another device is
 * current or the context is unusable.
 */
#define SLOWMO_STATIC_MAX_POINTERS 65536
slowmo_status slowmo_debias_static(slowmo_ctx *ctx, float *const *z, void *stream);

/*
 * The two learning-rate schedules of the paper's experiments, as functions of
 * the base-optimizer step number `step` >= 0 (the caller passes the result as
 * `lr`; nothing in a context depends on them).  Host-only, computed in double
 * precision and rounded once to float.
 *
 * slowmo_lr_step_decay (Section 4, CIFAR-10 and ImageNet): linear warm-up from
 * start_lr at step 0 to base_lr at step warmup_steps, then
 * base_lr * factor^(number of milestones <= step); the paper uses factor 0.1
 * at epochs 100/150/175 and 30/60/80 after 5 epochs of warm-up (the caller
 * converts epochs to steps).  milestones: n_milestones ascending step numbers
 * (may be NULL if n_milestones = 0).
 *
 * slowmo_lr_inverse_sqrt (Appendix A.3, WMT'16 En-De): linear warm-up from
 * init_lr to peak_lr over warmup_steps steps (4000 steps to 1e-3 in the
 * paper), then peak_lr * sqrt(warmup_steps / step).
 *
 * Errors: ARG for a NULL lr_out, step < 0, warmup_steps < 0, rates that are
 * not finite or base_lr / peak_lr <= 0, start_lr / init_lr < 0, factor not in
 * (0, 1], milestones that do not ascend.
 */
slowmo_status slowmo_lr_step_decay(float base_lr, float start_lr, int64_t warmup_steps,
                                   const int64_t *milestones, int32_t n_milestones, float factor,
                                   int64_t step, float *lr_out);
slowmo_status slowmo_lr_inverse_sqrt(float peak_lr, float init_lr, int64_t warmup_steps,
                                     int64_t step, float *lr_out);

/*
 * The communication pattern of Appendix C.1 (one-peer, time-varying directed
 * exponential graph): at iteration `step` every worker receives from the
 * worker 2^(step mod L) ranks below it (mod m), L = floor(log2(m-1)) + 1.
 * Writes the m entries of in_peer (host).  Host-only.  Errors: ARG.
 */
slowmo_status slowmo_expgraph_in_peers(int32_t m, int64_t step, int32_t *in_peer);

/*
 * Per-tensor hyper-parameters ("parameter groups").  The paper uses one
 * weight decay and one gamma_t for all parameters; this lets tensor j use
 *   weight decay weight_decay[j] instead of cfg.weight_decay, and
 *   the fast learning rate lr * lr_scale[j] wherever gamma_t acts on its
 *   elements: the local steps, Eq. (2) and Eq. (3) (so u stays in gradient
 *   units for every tensor, as Section 2 intends).
 * Host arrays of n_tensors entries; either may be NULL (left unchanged).
 * Applies to all later calls.  Synchronizes `stream`.
 * Errors: ARG (weight decay negative or non-finite, scale <= 0 or non-finite), HIP.
 */
slowmo_status slowmo_set_tensor_hparams(slowmo_ctx *ctx, const float *weight_decay,
                                        const float *lr_scale, void *stream);

/*
 * Checkpointing.  The optimizer's state is x0, u, h (and v), the counters
 * t, k, l and the push-sum weights; slowmo_export_state packs it into one DEVICE buffer of
 * slowmo_export_bytes() bytes (a 256-byte header, the push-sum weights, then the arrays), which the
 * caller may copy anywhere; slowmo_import_state restores it into a context
 * created with the same configuration and tensor list (otherwise ARG).  The
 * replicas themselves belong to the caller and are not part of the blob; as
 * slowmo_create overwrites replicas 1..m-1, restore them AFTER create when
 * resuming inside an outer iteration.  Per-tensor hyper-parameters are
 * configuration, not state: set them again.  Both calls synchronize `stream`.
 * Import checks the whole header and the weights before it touches the
 * context, then copies the arrays, waits for `stream`, and only then takes over
 * the counters and weights.
 * Errors: ARG, NOMEM (destination too small), HIP.
 */
size_t slowmo_export_bytes(const slowmo_ctx *ctx);
slowmo_status slowmo_export_state(slowmo_ctx *ctx, void *dst_device, size_t bytes, void *stream);
slowmo_status slowmo_import_state(slowmo_ctx *ctx, const void *src_device, size_t bytes,
                                  void *stream);

/*
 * Host-side check that [ptr, ptr + bytes) is memory the current device can
 * access: both ends known to the HIP runtime as device, managed or pinned host
 * memory of the current device, and inside one allocation where the runtime
 * can tell.  Launches nothing.  slowmo_create applies it to every parameter
 * tensor and to the workspace, so that a host pointer passed by mistake is an
 * ARG error instead of a GPU memory fault.  Environment variable
 * SLOWMO_CHECK_POINTERS, read at slowmo_create: 0 = no such checks, 1
 * (default) = at create, 2 = also the gradient tensors whenever their pointer
 * table changes and the destinations of slowmo_debias (a few microseconds per
 * tensor).  Errors: ARG (with the reason in slowmo_last_error(NULL)), HIP.
 */
slowmo_status slowmo_check_device_range(const void *ptr, size_t bytes);

/* Frees the context's host memory and its small device-side bookkeeping.
 * Never touches parameters, gradients or the workspace.  NULL is accepted. */
slowmo_status slowmo_destroy(slowmo_ctx *ctx);

/* Message of the last failed call on ctx; with ctx == NULL, of the last
 * failed call on this thread that had no context (e.g. a failed create).
 * Never NULL.  The string stays valid until the next call on that context
 * (or thread). */
const char *slowmo_last_error(const slowmo_ctx *ctx);

/*
 * Inspection (tests, checkpointing): device pointer to the first element of
 * an internal buffer of `tensor`: x0 / u (worker ignored, unless cfg.no_average
 * gave every worker its own), h / v of `worker`.
 * The numel[tensor] elements are contiguous.  Under the RESET policy h and v
 * are undefined from the last local step of an outer iteration (whose buffer
 * values nothing reads again, so they are not stored) until the next local
 * step.  ARG if the
 * buffer does not exist (v without Adam) or an index is out of range.
 */
slowmo_status slowmo_get_buffer(slowmo_ctx *ctx, int32_t which, int32_t worker, int32_t tensor,
                                float **device_ptr);

/* Counters: t = outer iterations completed, k = local steps taken in the
 * current outer iteration, l = Adam steps counted by the bias correction.
 * Any output pointer may be NULL. */
slowmo_status slowmo_get_counters(const slowmo_ctx *ctx, int64_t *t, int32_t *k, int64_t *l);

/*
 * Host-only view of the tiling (tests of the host logic; needs no device).
 * One record per tile: the contiguous run of elements of one tensor that one
 * workgroup processes.  The local-step tiling covers every (worker, tensor,
 * element) exactly once; the outer-step tiling covers every (tensor, element)
 * exactly once (worker = -1).  Tiles start at element offsets that are
 * multiples of 4, so a tile is 16-byte aligned whenever its tensor is.
 * Writes at most `cap` records to `out` (may be NULL with cap 0) and returns
 * the total number of records, or -1 on invalid arguments.
 */
typedef struct {
  int32_t tile;    /* index of the tile in launch order */
  int32_t worker;  /* -1 for the outer step */
  int32_t tensor;
  int32_t n;       /* elements in the run */
  int64_t offset;  /* first element of the run inside its tensor */
} slowmo_plan_run;

int64_t slowmo_plan_local(int32_t m, int32_t n_tensors, const int64_t *numel,
                          slowmo_plan_run *out, int64_t cap);
int64_t slowmo_plan_outer(int32_t m, int32_t n_tensors, const int64_t *numel,
                          slowmo_plan_run *out, int64_t cap);

/* Library version, e.g. "0.1.0 gfx950". */
const char *slowmo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SLOWMO_H */
