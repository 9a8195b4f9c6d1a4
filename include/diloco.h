/* diloco.h -- C ABI of the MI355X (gfx950) DiLoCo optimizer hot path.
 *
 * The method (OpenDiLoCo, arxiv 2407.07852, Section "Implementation" and Figure 1): k workers
 * each hold a replica of the model and run an inner optimizer (AdamW) for H local steps; then
 * an outer optimizer (SGD with Nesterov momentum) is applied to the weights theta(t) all
 * workers started the round from, using as its gradient the average over workers of the
 * pseudo-gradients  delta_r = theta(t) - theta_r(t+H).  Every worker then restarts from the
 * new outer weights.  Pseudo-gradients are FP32, optionally FP16 (Section "All-Reduce in
 * FP16").  With FP16 mixed precision a gradient scaler acts in the inner step only
 * (Section "Implementation", paragraph "General Implementation Details").
 *
 * Here all k replicas live on ONE GPU in a single caller-owned arena of flat, padded
 * multi-tensor buffers, and each step is one fused streaming kernel:
 *
 *   arena (FP32 slots):  theta0  mom  theta[k]  m[k]  v[k]  grads[k]     (buffer-major), or
 *                        theta0  mom  { theta_r  m_r  v_r  grads_r } x k  (worker-major)
 *   (n_pad <= slot elements of each buffer are used; see diloco_layout)
 *
 * theta0 = outer weights theta(t); mom = outer momentum buffer; theta/m/v = each worker's
 * weights and AdamW moments; grads = a place for each worker's gradients next to its state
 * (a caller may use it or pass its own buffer).  Every tensor of the parameter list starts at a multiple of 64
 * elements inside each buffer; the gaps and the tail up to n_pad hold zeros, and stay zero as
 * long as the gradient buffers hold zeros there too (both steps map 0 to 0).
 *
 * Conventions
 *   - "device" pointers are GPU global memory; "host" pointers are ordinary process memory.
 *   - The caller owns every large allocation (arena, gradients, flags).  The library borrows
 *     them.  Of its own it allocates 40*k bytes of device memory at diloco_init (per-worker
 *     step state and the per-step table) and, only if diloco_set_param_groups is used,
 *     n_pad/64 bytes more; the other entry points allocate nothing.
 *   - Every call returns DILOCO_OK (0), a positive informational code, or a negative error.
 *     On an error nothing has been launched.  No exception or abort crosses this boundary.
 *   - All device work is enqueued asynchronously on the stream given at init.
 *   - One context may be used by one host thread at a time.
 *   - The library fails loudly (DILOCO_ERR_HIP) when no usable GPU runtime is present; there
 *     is no CPU fallback.
 */
#ifndef DILOCO_H
#define DILOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct diloco_ctx diloco_ctx; /* opaque, host side */

enum {
  DILOCO_OK = 0,
  DILOCO_ROUND_COMPLETE = 1,       /* informational: the H-th inner step since the last outer step */
  DILOCO_ERR_INVALID_ARG = -1,     /* NULL, zero sizes, unknown dtype, hyper-parameter out of range */
  DILOCO_ERR_ALIGN = -2,           /* a device pointer or stride is not aligned for 128-bit access */
  DILOCO_ERR_ARENA_TOO_SMALL = -3, /* arena_bytes below what diloco_query_layout reports */
  DILOCO_ERR_HIP = -4,             /* the HIP runtime reported an error (also: asynchronous faults) */
  DILOCO_ERR_STATE = -5            /* call sequence error (e.g. flags passed without a check) */
};

enum { DILOCO_F32 = 0, DILOCO_F16 = 1, DILOCO_BF16 = 2 }; /* pseudo-gradient types; gradients: F32 or F16 */

enum { /* diloco_get_buffer selector */
  DILOCO_BUF_THETA0 = 0, /* outer weights theta(t), [n_pad] */
  DILOCO_BUF_MOM = 1,    /* outer Nesterov momentum buffer, [n_pad] */
  DILOCO_BUF_THETA = 2,  /* worker weights, replica r at + r*stride */
  DILOCO_BUF_M = 3,      /* AdamW first moment */
  DILOCO_BUF_V = 4,      /* AdamW second moment */
  DILOCO_BUF_GRADS = 5   /* the arena's gradient slot of replica r (FP32-sized; see diloco_layout) */
};

enum { /* diloco_config.layout_mode: order of the flat buffers inside the arena */
  DILOCO_LAYOUT_AUTO = 0,         /* by buffer size, see diloco_layout */
  DILOCO_LAYOUT_BUFFER_MAJOR = 1, /* theta0, mom, theta[k], m[k], v[k], grads[k] */
  DILOCO_LAYOUT_WORKER_MAJOR = 2  /* theta0, mom, then per worker: theta_r, m_r, v_r, grads_r */
};

#define DILOCO_MAX_WORKERS 64
#define DILOCO_MAX_GROUPS 8
#define DILOCO_TENSOR_ALIGN 64u /* elements: every tensor starts on a 256-byte boundary */
#define DILOCO_TILE 8192u       /* elements: n_pad is a multiple of this */
#define DILOCO_STRIDE_ALIGN_BYTES 2097152u /* stride*4 is a multiple of this (2 MiB) */

/* Problem statement: the parameter tensor list, the two optimizers' hyper-parameters
 * (Appendix A, Table 3 gives inner lr 4e-4, weight decay 0.1, outer lr 0.7, outer momentum
 * 0.9; betas and eps are not printed by the paper), H, k and the pseudo-gradient type. */
typedef struct {
  uint32_t n_tensors;       /* >= 1 */
  const uint64_t* numel;    /* host array [n_tensors], each >= 1, sum <= 2^33; copied at init */
  uint32_t k_workers;       /* 1 .. DILOCO_MAX_WORKERS */
  uint32_t h_inner_steps;   /* H; only used to report DILOCO_ROUND_COMPLETE; 0 = never */
  double inner_lr;          /* AdamW: >= 0, finite */
  double beta1, beta2;      /* in [0, 1) */
  double eps;               /* > 0 */
  double weight_decay;      /* >= 0 (decoupled) */
  double outer_lr;          /* Nesterov SGD: >= 0, finite */
  double outer_momentum;    /* in [0, 1) */
  int32_t pg_dtype;         /* DILOCO_F32, or DILOCO_F16 / DILOCO_BF16: round each worker's
                               pseudo-gradient to IEEE binary16 / bfloat16 (nearest-even,
                               subnormals kept, overflow to inf) and widen it back before the
                               FP32 average */
  int32_t pg_round_mean;    /* 0: the average stays FP32 (default).  1: the average is rounded
                               through pg_dtype as well, as the output of an all-reduce whose
                               buffer has that type would be (no effect with DILOCO_F32) */
  void* arena;              /* device, caller-owned, 256-byte aligned (2 MiB alignment, which large
                               allocations have anyway, is what the layout's stride assumes for
                               best bandwidth); unused by query_layout */
  uint64_t arena_bytes;
  void* stream;             /* hipStream_t, borrowed; NULL = the default stream */
  int32_t layout_mode;      /* DILOCO_LAYOUT_*; 0 = automatic */
  int32_t reserved;         /* 0 */
} diloco_config;

/* Where the flat buffers lie in the arena.  Every buffer occupies one slot of `slot` elements
 * (n_pad rounded up to 2 MiB); replica r of theta, m, v and of the arena's gradient slots
 * starts r*stride elements after replica 0.
 *   buffer-major: stride = slot; theta0, mom, theta[0..k), m[0..k), v[0..k), grads[0..k).
 *   worker-major: stride = 4*slot; theta0, mom, then theta_r, m_r, v_r, grads_r per worker.
 * The automatic choice is worker-major when a slot holds 2 GiB or more (about 0.54 billion
 * parameters per replica) or the whole arena exceeds 64 GiB, buffer-major otherwise: measured on MI355X, the inner step sustains
 * most when a worker's four streams are adjacent (1.6 to 3 points for such slots), and the outer
 * step when consecutive workers' weights lie 12-20 GiB apart or, when they are small, directly
 * adjacent.  Results never depend on the mode.
 * The gradient slots are FP32-sized; a caller may write gradients there (FP32: [k] rows of
 * n_pad floats, `stride` floats apart; binary16: rows of n_pad halves, 2*stride halves apart)
 * or pass any other device buffer to diloco_inner_step. */
typedef struct {
  uint64_t n_pad;       /* padded elements per flat buffer (multiple of DILOCO_TILE) */
  uint64_t stride;      /* elements between consecutive replicas of theta / m / v / grads */
  uint64_t arena_bytes; /* bytes the arena must provide */
  uint64_t off_theta0, off_mom, off_theta, off_m, off_v; /* byte offsets inside the arena */
  uint64_t off_grads;   /* byte offset of replica 0's gradient slot */
  uint64_t slot;        /* elements per buffer slot (>= n_pad) */
  int32_t layout_mode;  /* the mode in effect: DILOCO_LAYOUT_BUFFER_MAJOR or _WORKER_MAJOR */
  int32_t reserved;
} diloco_layout;

/* Flat layout for cfg's tensor list and k (host only, touches no GPU): the per-tensor iteration
 * of Figure 1 (`for param in model.parameters()`) becomes one pass over flat buffers; the two
 * model copies of paragraph "General Implementation Details" are theta0 and theta.
 * tensor_offsets may be NULL; otherwise it receives n_tensors element offsets, valid inside
 * every flat buffer (and inside the caller's gradient buffers).
 * Errors: DILOCO_ERR_INVALID_ARG (NULL, no tensors, an empty tensor, k out of range, more than
 * 2^33 parameters). */
int diloco_query_layout(const diloco_config* cfg, diloco_layout* out, uint64_t* tensor_offsets);

/* Creates a context over cfg->arena.  init_params: host array of n_tensors DEVICE pointers to
 * FP32 tensors that are packed into theta0; or NULL when theta0 in the arena already holds the
 * flat padded weights.  Then (Figure 1's starting state: every worker starts from the same
 * weights, `original_params` is a copy of them) every worker's weights are set to theta0,
 * moments and the outer momentum buffer to zero, step counts to zero; pads are zeroed.
 * *out is set only on success.  Errors: DILOCO_ERR_INVALID_ARG (problem or hyper-parameters out
 * of range, a pointer that is not memory of the current device or does not fit its
 * allocation), DILOCO_ERR_ALIGN, DILOCO_ERR_ARENA_TOO_SMALL, DILOCO_ERR_HIP. */
int diloco_init(const diloco_config* cfg, const void* const* init_params, diloco_ctx** out);

/* Gradient-scaler support for the inner step (mixed precision; Section "Implementation",
 * paragraph "General Implementation Details": the scaler acts in the inner step only).
 * grads: device, [k][grad_stride] elements of grad_dtype (DILOCO_F32 or DILOCO_F16), laid out
 * like the flat buffers; the pads must hold zeros (a non-finite pad would raise the flag, a
 * non-zero finite pad would move the pads of theta, m and v away from zero).  Sets found_inf[r]
 * (device, k int32) to 1 if any element of worker r's gradient is +-inf or NaN, else 0, and
 * records inv_scale (finite, > 0) as the factor the next diloco_inner_step applies to these
 * gradients, whatever their type.  The gradients are not modified: the multiply is fused into
 * the inner step.  Enqueues two kernels (flag clearing, check) and no memset.
 * Errors: DILOCO_ERR_INVALID_ARG, DILOCO_ERR_ALIGN, DILOCO_ERR_HIP. */
int diloco_unscale_check(diloco_ctx* ctx, const void* grads, uint64_t grad_stride,
                         int32_t grad_dtype, float inv_scale, int32_t* found_inf);

/* The inner optimizer step of Section "Implementation" (AdamW; `inner_optimizer.step()` in
 * Figure 1) for all k workers at once:
 *   g = grad (* inv_scale when found_inf is given)
 *   m = beta1*m + (1-beta1)*g ;  v = beta2*v + (1-beta2)*g*g
 *   theta = theta - lr*wd*theta - lr * (m/(1-beta1^t)) / (sqrt(v/(1-beta2^t)) + eps)
 * with t the worker's own step count.  grads as in diloco_unscale_check (grad_stride >= n_pad,
 * a multiple of 8 elements; base 16-byte aligned).  lr < 0 selects cfg->inner_lr.
 * found_inf: NULL, or the device flags written by the preceding diloco_unscale_check of the
 * same gradient buffer (else DILOCO_ERR_STATE); a worker whose flag is set skips the step: its
 * weights, moments and step count stay untouched.  DILOCO_F16 gradients exist only under a loss
 * scale, so they REQUIRE found_inf (DILOCO_ERR_STATE without it: they are never stepped
 * unchecked and unscaled).  Returns DILOCO_ROUND_COMPLETE on every H-th call since the last
 * outer step (a host-side count of calls: replays of a captured graph are not counted).
 * Stream capture: the call enqueues exactly two kernels and no memset -- a one-wave prologue that
 * advances every worker's step count and running beta^t products in place on the device (or
 * marks the worker inactive) and the AdamW kernel that reads the prologue's table.  The step
 * state lives on the device only, so a captured sequence with any number of inner steps, odd
 * included, replays correctly and can be mixed with eager calls.
 * The gradient buffer's extent is checked against its allocation when the pointer is first
 * passed; calls that repeat the last validated pointer (the steady state of a training loop)
 * skip the two runtime queries, so a buffer freed and re-allocated smaller at the same address
 * between two calls is the caller's responsibility.
 * Errors: DILOCO_ERR_INVALID_ARG, DILOCO_ERR_ALIGN, DILOCO_ERR_STATE, DILOCO_ERR_HIP. */
int diloco_inner_step(diloco_ctx* ctx, const void* grads, uint64_t grad_stride,
                      int32_t grad_dtype, double lr, const int32_t* found_inf);

/* Per-worker AdamW step state as diloco_inner_step_noalloc keeps it in caller memory: the running
 * products beta1^t and beta2^t and the step count t.  A fresh worker is {1.0, 1.0, 0, 0}. */
typedef struct {
  double beta1_pow;
  double beta2_pow;
  int32_t step;
  int32_t reserved; /* 0 */
} diloco_step_state;

/* Arguments of diloco_inner_step_noalloc.  All pointers are DEVICE pointers owned by the caller;
 * the struct itself is host memory, read during the call only. */
typedef struct {
  float* theta;                  /* worker 0's weights; worker r at + r*stride; in/out */
  float* m;                      /* AdamW first moments, same spacing; in/out */
  float* v;                      /* AdamW second moments, same spacing; in/out */
  uint64_t stride;               /* elements between workers, >= n_pad, multiple of 4 */
  uint64_t n_pad;                /* elements per worker, a positive multiple of DILOCO_TILE */
  uint32_t k_workers;            /* 1 .. DILOCO_MAX_WORKERS */
  int32_t grad_dtype;            /* DILOCO_F32 or DILOCO_F16 */
  const void* grads;             /* [k][grad_stride] gradients, 16-byte aligned */
  uint64_t grad_stride;          /* >= n_pad, multiple of 8 */
  float inv_scale;               /* factor applied to every gradient element (1.0 = none) */
  const int32_t* found_inf;      /* k flags, or NULL; a flagged worker takes no step */
  diloco_step_state* step_state; /* [k], in/out, 8-byte aligned */
  double lr, beta1, beta2, eps, weight_decay;
  void* stream;                  /* hipStream_t; NULL = the default stream */
} diloco_inner_call;

/* diloco_inner_step for callers that cannot allocate device memory at all -- code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc -- and therefore cannot
 * create a context either (diloco_init allocates the step state and the per-step table).  Same
 * kernels, same arithmetic and same results as diloco_inner_step with a single parameter
 * group; the caller passes every input and output explicitly, including the per-worker step
 * state, and the per-step table that the prologue kernel writes for the AdamW kernel lives in a
 * static device array inside the library (1 KiB per GPU, DILOCO_MAX_WORKERS entries).
 * The call allocates nothing, on the device or on the host, and enqueues two kernels on
 * `stream` of the current device.  k_workers above DILOCO_MAX_WORKERS is rejected with
 * DILOCO_ERR_INVALID_ARG.  All calls on one GPU share the one static table: calls whose kernels
 * may overlap on the same GPU (different streams, different threads) race and must be
 * serialised by the caller; nothing needs clearing between calls, each call overwrites the
 * entries it reads.  Pointer extents are NOT checked against their allocations (that would cost
 * runtime queries); NULL, alignment, sizes and hyper-parameter ranges are.
 * Errors: DILOCO_ERR_INVALID_ARG, DILOCO_ERR_ALIGN, DILOCO_ERR_STATE (DILOCO_F16 gradients
 * without found_inf), DILOCO_ERR_HIP; message via diloco_last_error(NULL). */
int diloco_inner_step_noalloc(const diloco_inner_call* call);

/* Per-tensor parameter groups for the inner optimizer: the paper prints one weight decay (0.1)
 * and one learning rate with 1000 warm-up steps (Appendix A, Table 3); training codes built on
 * the paper's framework commonly exempt norm and embedding tensors from decay, which is what
 * groups are for.  group_of_tensor: host array [n_tensors], values < n_groups;
 * lr_scale, weight_decay: host arrays [n_groups] (finite, >= 0).  From the next inner step on,
 * every element of a tensor of group g is stepped with learning rate lr*lr_scale[g] and weight
 * decay weight_decay[g]; cfg->weight_decay is then unused.  n_groups = 0 (pointers ignored)
 * restores the single group of the config.  1 <= n_groups <= DILOCO_MAX_GROUPS otherwise.
 * Allocates n_pad/64 bytes of device memory (one group id per 64-element chunk), freed at
 * destroy; synchronises the stream. */
int diloco_set_param_groups(diloco_ctx* ctx, const uint8_t* group_of_tensor, uint32_t n_groups,
                            const double* lr_scale, const double* weight_decay);

/* Learning-rate schedule, host arithmetic only (the result is what a caller passes as `lr` to
 * diloco_inner_step): linear warm-up from 0 over warmup_steps ("Number of warmup steps 1,000",
 * Table 3); then, when total_steps > warmup_steps, a half-cosine from base_lr down to
 * base_lr*final_ratio reached at total_steps and held afterwards; total_steps = 0 keeps base_lr
 * (the paper does not state a decay shape).  Returns NaN on invalid arguments (non-finite or
 * negative base_lr / final_ratio). */
double diloco_lr_at(uint64_t step, uint64_t warmup_steps, uint64_t total_steps, double base_lr,
                    double final_ratio);

/* The outer step of Figure 1 (pseudo-gradient, `all_reduce(op=AVG)` over the workers, reset,
 * `outer_optimizer.step()` = SGD with Nesterov momentum, re-snapshot; hyper-parameters of
 * Appendix A, Table 3; reduced-precision variant of Section "All-Reduce in FP16"), fused into
 * one launch:
 *   delta_r = theta0 - theta_r            (optionally rounded through binary16 / bfloat16)
 *   dbar    = (delta_0 + ... + delta_{k-1}) / k        (FP32, workers in ascending order;
 *                                                       rounded too when pg_round_mean is set)
 *   mom     = mu*mom + dbar ;  theta0 = theta0 - outer_lr*(dbar + mu*mom)
 *   theta_r = theta0 for every r.
 * AdamW moments and step counts are not touched.  Legal after any number of inner steps,
 * including none.  The gradient scaler plays no part here, and non-finite pseudo-gradients
 * propagate as IEEE arithmetic dictates.  Enqueues one kernel.  Errors: DILOCO_ERR_HIP. */
int diloco_outer_step(diloco_ctx* ctx);

/* Delayed application of the outer step: the asynchronous weight averaging, interleaved with the
 * next round's computation, that the paper's Conclusion (and the last sentence of Section
 * "Globally Distributed Training Setting") names as future work.  The paper gives no update
 * rule; the one implemented:
 *   diloco_outer_begin   at the round boundary copies every worker's weights into `snapshot`
 *                        (sigma_r) on the context's stream, then computes on `side_stream`, from
 *                        the snapshot, exactly what diloco_outer_step computes from the live
 *                        weights -- pseudo-gradients theta0 - sigma_r, rounding, average, Nesterov
 *                        step on theta0 and mom -- but resets no worker;
 *   diloco_inner_step    may be called any number of times in between: the update touches
 *                        theta0, mom and the snapshot only, so it can run at the same time;
 *   diloco_outer_finish  makes the context's stream wait for the update and applies it:
 *                        theta_r <- theta0_new - (sigma_r - theta_r) for every worker, which
 *                        carries each worker's progress since the snapshot over to the new
 *                        outer weights.
 * With no inner step in between, the pair equals diloco_outer_step bit for bit (finite weights).
 * snapshot: device, caller-owned, k rows of n_pad floats, `slot` floats apart (dense, whatever
 * the arena's layout mode; snapshot_bytes >= ((k-1)*slot + n_pad)*4), 16-byte aligned, untouched
 * by the caller until diloco_outer_finish has run.  side_stream: hipStream_t of the same
 * device (default priority); it may be the context's own stream, in which case nothing overlaps.  Between begin and finish
 * theta0 and mom are in flux: diloco_outer_step and a second diloco_outer_begin return
 * DILOCO_ERR_STATE, and so does diloco_outer_finish without a begin.  begin enqueues two
 * kernels and two event operations, finish one kernel and one; none allocates.
 * Errors: DILOCO_ERR_INVALID_ARG, DILOCO_ERR_ALIGN, DILOCO_ERR_STATE, DILOCO_ERR_HIP. */
int diloco_outer_begin(diloco_ctx* ctx, void* snapshot, uint64_t snapshot_bytes, void* side_stream);
int diloco_outer_finish(diloco_ctx* ctx);

/* Device address of a flat buffer (replica ignored for THETA0 / MOM): the two model copies and
 * the optimizer states of paragraph "General Implementation Details", e.g. to view a worker's
 * parameter tensors in place at tensor_offsets; DILOCO_BUF_GRADS is the arena's gradient slot
 * of that worker, which diloco_init leaves as it finds it (a caller that uses it clears the
 * pads once).  Errors: DILOCO_ERR_INVALID_ARG. */
int diloco_get_buffer(diloco_ctx* ctx, int which, uint32_t replica, void** dev_ptr);

/* The layout this context was created with (same values as diloco_query_layout).
 * Errors: DILOCO_ERR_INVALID_ARG (NULL). */
int diloco_get_layout(diloco_ctx* ctx, diloco_layout* out);

/* Per-worker AdamW step counts t_r into the host array steps[k]: a worker's count advances only
 * when its step is taken (a step skipped by the scaler is an optimizer step that was not
 * called; "General Implementation Details").  Synchronises the stream.
 * Errors: DILOCO_ERR_INVALID_ARG, DILOCO_ERR_HIP. */
int diloco_get_steps(diloco_ctx* ctx, uint32_t* steps);

/* DIAGNOSTIC, not part of the training path: the pseudo-gradient's FP32 -> binary16 / bfloat16
 * rounding on its own, with the same hardware conversion the outer step applies (Section
 * "All-Reduce in FP16"): in/out are device arrays of n elements (out: uint16 codes). */
int diloco_cast_f32_to_f16(const float* in, uint16_t* out, uint64_t n, void* stream);
int diloco_cast_f32_to_bf16(const float* in, uint16_t* out, uint64_t n, void* stream);

/* DIAGNOSTIC: launch-shape knobs for benchmarking sweeps; results never depend on them.  Names
 * and values:
 *   inner_block 64|128|256, outer_block -1|64|128|256 (threads per workgroup; -1 automatic),
 *   inner_waves / outer_waves -1..32 (resident waves per CU: -1 automatic, 0 hardware maximum),
 *   outer_anyk 0|1 (1: the run-time-k kernel also for k <= 8),
 *   snapshot_waves / update_waves / merge_waves -1..32 (the delayed outer step's three kernels),
 *   check_block 64|256, check_vec 1|2|4|8, check_waves 0..32, check_persist 0..64.
 * The defaults are the measured optimum on MI355X.  Unknown names or values return
 * DILOCO_ERR_INVALID_ARG. */
int diloco_set_tuning(diloco_ctx* ctx, const char* name, int value);

/* Message of the most recent error on this context (ctx may be NULL: the calling thread's
 * last error from diloco_init / diloco_query_layout).  Never NULL. */
const char* diloco_last_error(diloco_ctx* ctx);

/* Synchronises the stream, frees the library's own device state and the host context.  The
 * arena and every caller buffer are left untouched.  NULL is accepted. */
int diloco_destroy(diloco_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif
