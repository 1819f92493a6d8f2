/*
 * dapple_stage.h -- C ABI of one pipeline stage of synchronous pipelined training
 * on one MI355X (gfx950).
 *
 * The stage is a stack of post-LayerNorm transformer encoder layers (optionally
 * preceded by an embedding block or followed by a masked-LM head).  It runs the
 * forward task F_m and the backward task B_m of M micro-batches in a forced
 * order with at most K micro-batches of activations resident, and accumulates
 * weight gradients in fp32 over all micro-batches of the iteration.
 *
 * Where each call comes from in the DAPPLE paper (arXiv 2007.01045):
 *   stage_fwd / stage_bwd   the per-stage forward / backward tasks F_s, B_s of one
 *                           micro-batch (section IV-A; stage graphs built forward
 *                           in order, backward in reverse, section V-A).
 *   stage_run_schedule      early backward scheduling (section III-B) and the
 *                           micro-batch unit scheduling rules (section V-C):
 *                           inject K micro-batches, then strictly alternate one
 *                           backward and one forward, the backward first so that
 *                           its activations are released before the next forward
 *                           reuses them; GPipe order (section III-A) for contrast.
 *   stage_grads /           gradient accumulation over all micro-batches of the
 *   stage_zero_grads        iteration on the device (section V-B-3).  The sum is
 *                           returned, not the average: averaging belongs to Apply.
 *   stage_stats             peak activation memory, the quantity Table VI reports.
 *
 * Conventions
 *   - every pointer named *_dev is DEVICE memory owned by the caller; every other
 *     pointer is HOST memory.  The library allocates no device memory: it
 *     sub-allocates the arena handed to stage_init (gradient accumulators,
 *     max_slots activation slots, workspace).
 *   - all device work is ordered in the HIP stream given to stage_init; no call
 *     synchronises the stream except stage_sync.  (The library owns up to three more
 *     streams: one for the gradient-accumulator kernels of every backward task, and,
 *     inside stage_run_schedule, one for the forward tasks and one for every second
 *     backward task.  All are forked from and joined back into the caller's stream
 *     inside the call, so the caller's stream order still covers everything.)
 *     Buffers passed to a call must stay valid until the stream has passed that call.
 *   - every call returns 0 on success or a negative STAGE_E_* code; nothing throws
 *     or aborts.  stage_last_error() gives a message for the last failure of the
 *     calling thread.  A call that fails with any code but STAGE_E_DEVICE has enqueued
 *     nothing and changed no state (arguments, orders and slot use are checked on the
 *     host first).  STAGE_E_DEVICE means a HIP call failed part-way: work may already
 *     be enqueued and micro-batches may be left resident; the only calls defined on
 *     such a handle are stage_sync and stage_destroy.
 *   - element type: dtype 0 = fp32 everywhere; dtype 1 = bf16 storage for
 *     weights, activations and boundary tensors with fp32 accumulation inside
 *     kernels and fp32 gradient accumulators.
 *   - linear weights are [in, out] row-major (y = x W + b).  Flat parameter order:
 *     embedding block (E_w[V,H], E_p[P,H], ln_g, ln_b) if present; per layer
 *     Wq,bq,Wk,bk,Wv,bv,Wo,bo,ln1_g,ln1_b,W1,b1,W2,b2,ln2_g,ln2_b; head block
 *     (Wt,bt,ln_g,ln_b,E_out[V,H],b_out[V]) if present.  Gradients use the same
 *     order, always fp32.
 */
#ifndef DAPPLE_STAGE_H
#define DAPPLE_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STAGE_OK = 0,
  STAGE_E_CONFIG = -1,       /* inconsistent or unsupported configuration */
  STAGE_E_NULL = -2,         /* a required pointer is NULL */
  STAGE_E_ARENA_SMALL = -3,  /* arena smaller than stage_query_sizes says */
  STAGE_E_NO_SLOT = -4,      /* forward while max_slots micro-batches are resident */
  STAGE_E_NOT_RESIDENT = -5, /* backward of a micro-batch with no live forward */
  STAGE_E_DUP_MB = -6,       /* forward of a micro-batch that is already resident */
  STAGE_E_BAD_ORDER = -7,    /* M < 1, K < 1, K > max_slots, or an invalid explicit list */
  STAGE_E_DEVICE = -8        /* a HIP call failed */
};

enum { STAGE_ORDER_GPIPE = 0, STAGE_ORDER_EARLY_BACKWARD = 1, STAGE_ORDER_EXPLICIT = 2 };
enum { STAGE_DTYPE_F32 = 0, STAGE_DTYPE_BF16 = 1 };
enum {
  STAGE_FLAG_DRY_RUN = 1,   /* host bookkeeping only: no kernel is launched and device pointers may
                               be NULL (for CPU-side tests) */
  STAGE_FLAG_RECOMPUTE = 2, /* re-computation (section VI-E, Table VI's "+ RC" rows): a resident
                               micro-batch keeps only the stage's input (token ids on a first stage)
                               and its targets; stage_bwd re-runs the forward from them before it goes
                               backward.  slot_bytes shrinks to that; activation buffers of the full
                               size -- one for the forward tasks and one per backward lane (two lanes;
                               one with STAGE_FLAG_ONE_STREAM) -- are part of the arena and of
                               peak_activation_bytes, whatever K and M are.  Gradients and outputs are
                               bit-identical to the stage without the flag. */
  STAGE_FLAG_ONE_STREAM = 4 /* every kernel goes on the stage's own stream: no library-owned lanes.
                               For a stage that is one of several run beside each other
                               (dapple_pipeline.h), where the overlap comes from the other stages and
                               every extra hardware queue costs.  Same bits as without the flag. */
};

typedef struct {
  int32_t n_layers, hidden, n_heads, ffn, seq, micro_batch; /* L, H, A, F, s, b */
  int32_t max_slots;     /* activation slots carved from the arena (K; M for GPipe order) */
  int32_t dtype;         /* STAGE_DTYPE_* */
  int32_t has_embedding; /* first stage: x is int32 token ids [b*s] */
  int32_t has_mlm_head;  /* last stage: y is float loss[1], aux is int32 targets [b*s] */
  int32_t vocab, max_pos;
  int32_t flags;         /* STAGE_FLAG_* */
  float ln_eps;          /* added to the biased variance inside the square root */
  float loss_scale;      /* MLM head: loss = loss_scale * sum over predicted rows */
  int32_t mlm_max_rows;  /* MLM head: most predicted positions per micro-batch (0 = all b*s rows);
                            sizes the head's buffers; more predicted rows than this are dropped and
                            stage_sync then returns STAGE_E_CONFIG */
} stage_config;

typedef struct {
  uint64_t n_params;        /* elements of the flat parameter / gradient vector */
  uint64_t weight_bytes;    /* bytes of the caller's flat parameter vector */
  uint64_t grad_bytes;      /* fp32 accumulators */
  uint64_t slot_bytes;      /* activations one resident micro-batch keeps from F to B */
  uint64_t workspace_bytes; /* transient buffers shared by all tasks (one copy) */
  uint64_t arena_bytes;     /* grad_bytes + max_slots * slot_bytes + copies * workspace_bytes (+ alignment, + the
                               forward tasks' activation buffer under STAGE_FLAG_RECOMPUTE); copies = 2 (one
                               workspace per backward lane), 1 under STAGE_FLAG_ONE_STREAM */
} stage_sizes;

typedef struct {
  uint64_t slot_bytes;
  uint64_t peak_activation_bytes; /* peak_live_slots * slot_bytes (+ the activation buffers of
                                     STAGE_FLAG_RECOMPUTE: forward tasks' + one per backward lane) */
  int32_t live_slots, peak_live_slots;
  uint64_t fwd_tasks, bwd_tasks, kernel_launches;
} stage_stats_t;

typedef struct dapple_stage* stage_handle;

/* Sizes for a configuration; host only, no device needed. */
int stage_query_sizes(const stage_config* cfg, stage_sizes* out);

/* Create a stage.  weights_dev: flat parameters (dtype of the config), read by every
 * task and never written; arena_dev: at least arena_bytes, 256-byte aligned;
 * hip_stream: a hipStream_t (NULL = the default stream).  Zeroes the accumulators. */
int stage_init(stage_handle* out, const stage_config* cfg, const void* weights_dev,
               void* arena_dev, size_t arena_bytes, void* hip_stream);

/* F_m.  x_dev [b*s, H] (or int32 ids [b*s]); y_dev [b*s, H] (or float loss[1]);
 * aux_dev: int32 targets [b*s], -1 = not predicted (MLM head only, else NULL).
 * Binds micro-batch mb to a free activation slot. */
int stage_fwd(stage_handle h, int mb, const void* x_dev, void* y_dev, const void* aux_dev);

/* B_m.  dy_dev [b*s, H] (NULL with the MLM head); dx_dev [b*s, H] (NULL with the
 * embedding block).  Adds this micro-batch's weight gradients into the fp32
 * accumulators and releases the slot. */
int stage_bwd(stage_handle h, int mb, const void* dy_dev, void* dx_dev);

/* Host-only: the task list of an order.  ops_out receives +(m+1) for F_m and
 * -(m+1) for B_m; returns the number of tasks (2M) or a negative error.
 * Early-backward: F_0..F_{K'-1}, then (B_j, F_{j+K'}) for j = 0..M-K'-1, then the
 * remaining backwards, K' = min(K, M).  Backwards ascend in both orders. */
int stage_schedule_ops(int M, int K, int order, int32_t* ops_out, int capacity);

/* Run one iteration's tasks in the given order on the stream.  xs, dys, ys, dxs,
 * auxs: host arrays of M device pointers (arrays that do not apply may be NULL).
 * order EXPLICIT takes explicit_ops/n_ops in the encoding above; the list is
 * validated (each F before its B, every micro-batch once, at most K resident)
 * before anything is enqueued.
 * The early-backward order is executed as the dependence graph that defines it
 * (the control edges B_m -> F_{m+K} of section V-C plus F_m -> B_m, forwards in
 * list order): forward tasks go to the library's forward stream, backward tasks
 * alternate between the caller's stream and a second backward stream (each with
 * its own workspace), and every gradient-accumulator update of every backward task
 * goes to the one side stream in list order, which fixes the order of every sum.
 * The GPipe order alternates its backward tasks the same way but starts none before
 * the last forward listed before it has finished; an explicit list keeps one backward
 * stream and the same rule.  Results do not depend on the overlap: they are the same
 * bits as with STAGE_FLAG_ONE_STREAM. */
int stage_run_schedule(stage_handle h, int M, int K, int order,
                       const void* const* xs, const void* const* dys,
                       void* const* ys, void* const* dxs, const void* const* auxs,
                       const int32_t* explicit_ops, int n_ops);

/* The same iteration as ONE HIP graph: stage_graph_capture records what stage_run_schedule would
 * enqueue (all of the library's streams, forked from and joined back into the caller's stream;
 * with zero_grads_first != 0 preceded by stage_zero_grads) and instantiates it; stage_graph_launch
 * replays it on the caller's stream at the cost of one launch call.  The device pointers of the
 * capture are baked in.  Requirements: the stage's stream is not the default (NULL) stream; the
 * same iteration ran eagerly once before (the kernels' launch attributes are set on their first
 * eager launch); no micro-batch is resident; per-launch timing is off.  The graph holds no memset
 * node (accumulators and buffers are cleared by kernels).  A new capture replaces the old one;
 * stage_destroy frees it.  Task and launch counters advance per replay as if run eagerly.
 * The captured iteration uses one backward lane (results are the same bits either way), and a
 * replay has measured no faster than the eager lanes: this pair is for callers that need the
 * iteration as one launchable object. */
int stage_graph_capture(stage_handle h, int M, int K, int order,
                        const void* const* xs, const void* const* dys,
                        void* const* ys, void* const* dxs, const void* const* auxs,
                        const int32_t* explicit_ops, int n_ops, int zero_grads_first);
int stage_graph_launch(stage_handle h);

/* The stream the stage was created on, and a copy of its configuration. */
int stage_stream(stage_handle h, void** hip_stream_out);
int stage_get_config(stage_handle h, stage_config* cfg_out);

/* Device pointer to the fp32 accumulators (aliases the arena; valid until
 * stage_destroy) and their element count. */
int stage_grads(stage_handle h, void** grads_dev, uint64_t* n);
int stage_zero_grads(stage_handle h);

/* The Apply of the synchronous weights update (section V-B-3) with the optimizer the paper
 * trains BERT-48 with (Adam, section VI-A; 16 bytes of fp32 state per parameter, Table VIII):
 * one fused pass over all parameters of the stage, to be called after the iteration's tasks.
 *   g = grad_scale * G (the averaging over the iteration's samples is the caller's choice),
 *   m = beta1 m + (1-beta1) g,  v = beta2 v + (1-beta2) g^2,
 *   master -= lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps),  step >= 1,
 *   weights = master rounded to the stage's dtype.
 * weights_dev: the buffer given to stage_init (it is written here and nowhere else);
 * master_dev, m_dev, v_dev: device fp32 [n_params], 16-byte aligned, owned by the caller
 * (master initialised to the weights, moments to zero).  zero_grads != 0 also clears the
 * accumulators in the same pass.  Fails with STAGE_E_BAD_ORDER while micro-batches are
 * resident. */
int stage_apply_adam(stage_handle h, void* weights_dev, float* master_dev, float* m_dev, float* v_dev,
                     int step, float lr, float beta1, float beta2, float eps, float grad_scale,
                     int zero_grads);

int stage_stats(stage_handle h, stage_stats_t* out);
int stage_reset_stats(stage_handle h);

/* Per-kernel-class timing with HIP events on the stage's stream.  While enabled
 * every launch is bracketed by two events; stage_profile_read synchronises the
 * stream and returns, for class i < n, launches[i], total milliseconds ms[i] and the
 * algorithmic flops[i] (multiply-add = 2) of those launches.  Class names:
 * stage_profile_class_name(i), NULL past the end. */
int stage_profile_enable(stage_handle h, int on);
int stage_profile_read(stage_handle h, int n, uint64_t* launches, double* ms, double* flops);
/* The launches timed since stage_profile_enable / the last stage_profile_read, one record each, in
 * the order they were enqueued (call it before stage_profile_read, which clears them): class,
 * stream (0 = caller's, 1 = side, 2 = forward, 3 = second backward), milliseconds, algorithmic
 * flops, and for matrix products M, N, K and the number of products in the launch (0 otherwise).
 * Synchronises the stage's streams.  Returns the number of records written (at most capacity). */
typedef struct {
  int32_t cls, lane;
  int32_t M, N, K, batch;
  double ms, flops;
} stage_launch_record;
int stage_profile_launches(stage_handle h, stage_launch_record* out, int capacity);
const char* stage_profile_class_name(int i);

int stage_sync(stage_handle h);
int stage_destroy(stage_handle h);
const char* stage_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
