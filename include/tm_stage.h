/*
 * tm_stage.h - C ABI of the stage-shard training step for AMD MI355X (gfx950).
 *
 * What the library runs.  TrainMover (arXiv 2412.12636) warms a joining
 * machine by letting it execute one full "shadow" training iteration of its
 * model partition inside a communication-free sandbox (section 4.2): state is
 * first loaded from a checkpoint, every tensor that would arrive from outside
 * the sandbox is supplied locally, `send` and `barrier` are skipped, and
 * afterwards all local state is overwritten by the leaver's (sections 4.2 and
 * 7).  For a middle pipeline stage the partition is a run of identical
 * transformer blocks on a tensor-parallel shard (section 6.1).  This library is
 * that iteration for one GPU: forward and backward through the stage's layers
 * with every tensor/pipeline-parallel collective acting as the identity,
 * followed by the mixed-precision Adam update of the shard.
 *
 * Consequences for the interface:
 *  - the two boundary tensors of a pipeline stage are arguments: `x` (what the
 *    previous stage would send) and `dy` (what the next stage would send back);
 *  - parameters, optimizer states and the gradient buffer (section 8.4 speaks
 *    of a pre-allocated gradient buffer) are flat, CALLER-OWNED device buffers
 *    that may be rewritten between any two calls; the library keeps no copies;
 *  - the library never allocates or frees device memory and never synchronises
 *    the device; it only enqueues kernels on the caller's stream.
 *
 * All sizes in the configuration are LOCAL to the rank (after the
 * tensor-parallel slice).  Activations are [seq, micro_batch, hidden]
 * row-major, i.e. token row t = position * micro_batch + batch_entry.
 *
 * Every function returns 0 (TM_OK) or a negative tm_status_t; none throws.
 * After a failure tm_last_error() holds a message.  A handle must not be used
 * from two threads at once; distinct handles are independent.
 */
#ifndef TM_STAGE_H
#define TM_STAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tm_stage tm_stage_t; /* opaque, lives in host memory */

typedef enum {
  TM_OK = 0,
  TM_EINVAL = -1,  /* NULL pointer or a value outside the documented range */
  TM_EALIGN = -2,  /* a device pointer is not 256-byte aligned */
  TM_ESIZE = -3,   /* a size the kernels do not support (see tm_stage_config_t) */
  TM_EARCH = -4,   /* the current device is not gfx950 */
  TM_ELAUNCH = -5, /* a kernel launch or stream operation reported an error */
  TM_ESTATE = -6   /* call order violated (bwd without fwd) */
} tm_status_t;

enum { TM_DTYPE_FP32 = 0, TM_DTYPE_BF16 = 1 };
enum { TM_NORM_LAYERNORM = 0, TM_NORM_RMSNORM = 1 };
enum { TM_ACT_GELU_TANH = 0, TM_ACT_GELU_ERF = 1, TM_ACT_SWIGLU = 2 };
enum { TM_POS_NONE = 0, TM_POS_ROTARY = 1 };

/*
 * Shape of one rank's stage.  Constraints (violations give TM_ESIZE):
 * hidden, head_dim and ffn are multiples of 8; hidden <= 16384 (bf16) or
 * 8192 (fp32); head_dim <= 256 and even; n_q_heads is a multiple of
 * n_kv_heads; seq * micro_batch < 2^31 / max row width.
 */
typedef struct {
  int32_t n_layers;
  int32_t hidden;
  int32_t n_q_heads;   /* local query heads */
  int32_t n_kv_heads;  /* local key/value heads (grouped-query attention when smaller) */
  int32_t head_dim;
  int32_t ffn;         /* local MLP width f; the first MLP matrix has 2f rows under SwiGLU ([gate; up]) */
  int32_t seq;
  int32_t micro_batch;
  int32_t dtype;       /* TM_DTYPE_FP32: everything fp32.  TM_DTYPE_BF16: bf16 parameters and
                          activations, fp32 accumulation, fp32 gradients / master weights / Adam states */
  int32_t norm;        /* TM_NORM_* ; LayerNorm has gain and offset, RMSNorm gain only */
  int32_t act;         /* TM_ACT_* */
  int32_t pos;         /* TM_POS_ROTARY rotates element j with element j + head_dim/2 of every q and k head */
  int32_t has_bias;    /* biases on the four linear maps */
  double norm_eps;
  double rope_theta;
} tm_stage_config_t;

/*
 * Device buffers, all caller-owned and 256-byte aligned.
 *   params      n = tm_stage_param_count() elements of the stage dtype, layout per tm_stage_param_layout
 *   master      n fp32 master weights (bf16 stages).  For fp32 stages pass NULL: params is the master.
 *   grads       n fp32 gradients, same element order.  tm_stage_bwd ADDS into it.
 *   exp_avg, exp_avg_sq   n fp32 Adam moments
 *   workspace   tm_stage_workspace_bytes() bytes: activation stash written by fwd and read by bwd,
 *               plus scratch.  Contents are private to the library between fwd and bwd.
 *   workspace_bytes   the size of that allocation; tm_stage_init refuses (TM_ESIZE) one that is smaller
 *               than tm_stage_workspace_bytes() of the same library build
 */
typedef struct {
  void *params;
  float *master;
  float *grads;
  float *exp_avg;
  float *exp_avg_sq;
  void *workspace;
  int64_t workspace_bytes;
} tm_stage_buffers_t;

typedef struct {
  double lr, beta1, beta2, eps;
  double weight_decay; /* decoupled (AdamW form); 0 = plain Adam */
  double grad_scale;   /* gradient is multiplied by this first (1/micro-batches, clipping factor, ...) */
  int32_t zero_grads;  /* non-zero: gradients are cleared after they are consumed */
} tm_adam_hparams_t;

/* Pure functions of the configuration (host only, no device needed).  Negative = tm_status_t. */
int64_t tm_stage_param_count(const tm_stage_config_t *cfg);
int64_t tm_stage_workspace_bytes(const tm_stage_config_t *cfg);

/*
 * Enumerates the parameter tensors in flat-buffer order.  index runs over
 * [0, tm_stage_param_layout(cfg, -1, ...)): a call with index -1 returns the
 * tensor count.  For index >= 0: *name points to a static string such as
 * "layer3.w_qkv", *offset_elems is the element offset in every flat buffer,
 * shape[0..1] the row-major shape (shape[1] = 1 for vectors).  Returns TM_OK
 * or TM_EINVAL.  Per layer, in order: norm1_gain, [norm1_offset], w_qkv
 * [(nq+2nkv)*d, h] with rows ordered Q heads, K heads, V heads, [b_qkv], w_out
 * [h, nq*d], [b_out], norm2_gain, [norm2_offset], w_fc1 [f or 2f, h], [b_fc1],
 * w_fc2 [h, f], [b_fc2].  All linear maps are y = x W^T + b.
 */
int tm_stage_param_layout(const tm_stage_config_t *cfg, int index, const char **name,
                          int64_t *offset_elems, int64_t shape[2]);

/*
 * Validates the configuration and the buffers and creates a handle (host
 * memory only).  The current HIP device must be gfx950 (else TM_EARCH).
 * Nothing is launched; buffer contents are not touched.
 */
int tm_stage_init(const tm_stage_config_t *cfg, const tm_stage_buffers_t *buffers, tm_stage_t **out);

/*
 * Optional, bf16 stages: measures the tile configurations of the matrix-core
 * GEMM kernel on the twelve products of this stage's shard shape (three per
 * linear map of the transformer block, section 6.1's per-rank share) and makes
 * every later product of those shapes, in this process, use the fastest.
 * Runs on `stream`, WAITS for it, and uses the workspace as operands and
 * results: call it before the first forward pass (a stash from an earlier
 * forward pass is invalidated: the next call must be tm_stage_fwd).  Without
 * it a cost model picks the configurations.  The choice changes speed only:
 * every configuration accumulates each output in the same order.
 */
int tm_stage_tune(tm_stage_t *st, void *stream);

/*
 * Forward pass of all layers (section 4.2: the forward half of the shadow
 * iteration; the pipeline receive is served by x_in).  x_in and y_out are
 * device pointers to [seq, micro_batch, hidden] tensors of the stage dtype,
 * 256-byte aligned; they may not alias each other or the workspace.  Reads
 * params at launch time.  stream is a hipStream_t (NULL = default stream).
 */
int tm_stage_fwd(tm_stage_t *st, const void *x_in, void *y_out, void *stream);

/*
 * Backward pass for the most recent tm_stage_fwd (the pipeline receive of the
 * output gradient is served by dy_in; sends are skipped).  Writes the input
 * gradient to dx_out and ADDS parameter gradients into buffers.grads.
 * TM_ESTATE if no forward pass precedes it.  Must be enqueued on the same
 * stream as that forward pass or after it has completed.
 */
int tm_stage_bwd(tm_stage_t *st, const void *dy_in, void *dx_out, void *stream);

/*
 * Gradient-buffer mode of the following tm_stage_bwd calls.  TM_GRAD_ADD (0, the default): parameter
 * gradients are ADDED into buffers.grads (gradient accumulation over micro-batches).  TM_GRAD_STORE (1):
 * they are STORED, the buffer's old contents are not read - for the first micro-batch of an iteration,
 * when those contents are dead; it saves one read of the fp32 gradient buffer per backward pass and
 * makes clearing the buffer unnecessary.  TM_GRAD_TRANSIENT (2): as TM_GRAD_STORE, and tm_stage_bwd_adam
 * may consume a gradient without storing it (where the update rides in a weight-gradient product, see
 * there): afterwards those entries of buffers.grads are unspecified - for iterations of one micro-batch
 * whose gradients nobody reads after the update.
 */
enum { TM_GRAD_ADD = 0, TM_GRAD_STORE = 1, TM_GRAD_TRANSIENT = 2 };
int tm_stage_grad_mode(tm_stage_t *st, int mode);

/*
 * Adam with bias correction at step >= 1 on the whole shard:
 *   g' = grad_scale*g;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2
 *   p -= lr*( (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps) + weight_decay*p )
 * on the fp32 master weights; bf16 stages also store round-to-nearest-even
 * copies into buffers.params.  (Optimizer step of the shadow iteration.)
 */
int tm_adam_step(tm_stage_t *st, const tm_adam_hparams_t *hp, int64_t step, void *stream);

/*
 * Backward pass plus optimizer step in one call, for the LAST micro-batch of an
 * iteration: the same results, bit for bit, as tm_stage_bwd followed by
 * tm_adam_step, but every layer's update is enqueued as soon as that layer's
 * gradients are complete.  Valid only when nothing global is
 * derived from this pass's gradients before the update: hp->grad_scale must
 * not depend on them (no norm-based clipping).  For bf16 stages in TM_GRAD_STORE
 * or TM_GRAD_TRANSIENT mode with hp->zero_grads == 0 and a token count that is a
 * multiple of 64, the update of each weight matrix is applied in the epilogue of
 * its weight-gradient product, from the accumulators (the gradient is not read
 * back; in TM_GRAD_TRANSIENT mode it is not stored either), and the flat sweep
 * covers the vectors between the matrices; the results are the same bits.  Everything is enqueued on
 * `stream`; with TM_BWD_STREAMS=2 in the environment the weight-gradient products and the updates go to
 * internal streams that are ordered after everything enqueued on `stream` so far, and `stream` waits for
 * them before the call's work counts as done.  (Shadow iteration, section 4.2:
 * the last steps of the iteration the sandbox replays.)
 */
int tm_stage_bwd_adam(tm_stage_t *st, const void *dy, void *dx, const tm_adam_hparams_t *hp,
                      int64_t step, void *stream);

/*
 * Pieces of a whole iteration as the paper's default profiles run it (section
 * 8.1: several micro-batches per iteration, distributed optimizer): after the
 * micro-batches' backward passes have added up in buffers.grads,
 *   tm_stage_grad_sq_sum  writes the sum of squares of all gradients of this
 *       rank (its contribution to the squared global norm; the sum over ranks
 *       is served locally) to out[0], a DEVICE double; fixed summation order;
 *       uses the workspace's scratch, so not between a forward pass and its
 *       backward pass's use of that scratch: call it after tm_stage_bwd;
 *   the caller forms hp->grad_scale from it (1/micro-batches times the clipping
 *       factor min(1, c / (norm + 1e-6)));
 *   tm_adam_step_range  updates elements [first, first+count) of the flat
 *       state only: this data-parallel rank's share under a distributed
 *       optimizer (first a multiple of 8; TM_EINVAL outside the state).
 */
int tm_stage_grad_sq_sum(tm_stage_t *st, double *out, void *stream);
int tm_adam_step_range(tm_stage_t *st, int64_t first, int64_t count, const tm_adam_hparams_t *hp,
                       int64_t step, void *stream);

/*
 * Sum of squares of n fp32 values (16-byte aligned) into out[0] (device
 * double), two passes in a fixed order; scratch: tm_sq_sum_scratch_bytes(n)
 * bytes, 8-byte aligned.
 */
int64_t tm_sq_sum_scratch_bytes(int64_t n);
int tm_sq_sum(int64_t n, const float *g, void *scratch, double *out, void *stream);

/*
 * tm_sq_sum for callers that cannot allocate device memory or hand over scratch (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same two kernels, same order, same
 * bits, with the block partials in a buffer built into the library (8 MiB per GPU, held by every GPU the
 * library runs on until the process ends).  n is at most tm_sq_sum_static_max_elems() = 2^32 elements
 * (TM_ESIZE beyond).  g and out are device pointers as in tm_sq_sum.  Allocates nothing, never
 * synchronises.  All calls on one GPU share that GPU's buffer: calls that overlap on one GPU (two streams,
 * two threads) race; calls ordered on one stream do not.  Nothing in the buffer has to survive or to be
 * cleared between calls.
 */
int64_t tm_sq_sum_static_max_elems(void);
int tm_sq_sum_static(int64_t n, const float *g, double *out, void *stream);

/*
 * The same update on bare flat device arrays of n elements (p, m, v updated in
 * place; g read, and cleared if hp->zero_grads; p_bf16 may be NULL).  This is
 * what a distributed-optimizer rank would call on its slice.  Pointers must be
 * 16-byte aligned.
 */
int tm_adam_step_flat(int64_t n, float *p, float *g, float *m, float *v, void *p_bf16,
                      const tm_adam_hparams_t *hp, int64_t step, void *stream);

void tm_stage_destroy(tm_stage_t *st);

/*
 * Optional per-kernel timing for measurement.  While enabled, every step that tm_stage_fwd,
 * tm_stage_bwd and tm_adam_step enqueue is bracketed by two HIP events on the caller's stream.
 * tm_stage_profile_collect waits for the recorded events (the only call here that blocks the
 * host), sums elapsed time, launch count and algorithmic work per kernel name into entries[]
 * (at most max_entries; `kernel` points at static storage), clears the record list and returns
 * the number of entries filled.  flops counts 2*M*N*K per matrix product and 2*b*nq*s^2*d per
 * causal attention forward (twice that backward); bytes counts the operands and results of the
 * streaming kernels once.  Disabling frees the events.  Events are host objects: no device
 * memory is allocated.
 */
typedef struct {
  const char *kernel;
  double ms;
  double flops;
  double bytes;
  int64_t launches;
} tm_profile_entry_t;
int tm_stage_profile_enable(tm_stage_t *st, int enable);
int tm_stage_profile_collect(tm_stage_t *st, tm_profile_entry_t *entries, int max_entries);

/* Message of the last failure on the calling thread; never NULL. */
const char *tm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TM_STAGE_H */
