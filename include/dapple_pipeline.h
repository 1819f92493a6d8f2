/* dapple_pipeline.h -- S pipeline stages of one GPU run as a pipeline: the micro-batch
 * unit scheduling of the DAPPLE paper (section V-C) across stages, for studying the
 * schedule (who waits for whom, how many micro-batches each stage keeps, where the
 * bubbles are) against the planner's latency model (section IV-A, equations 1 and 2).
 *
 * Every stage is a dapple_stage (dapple_stage.h) with a stream of its own.  Stage i runs
 * its own task list -- K_i forwards, then one backward / one forward in turn, then the
 * remaining backwards -- in list order on its stream (the control edges of section V-C);
 * across stages a HIP event per task carries the data edges: F_{i,m} waits for
 * F_{i-1,m}, B_{i,m} for B_{i+1,m}; the boundary activation and its gradient go through
 * a buffer the caller provides (on one GPU the "transfer" of section V-A is the buffer
 * itself).  To let the stages run beside each other like devices of their own, a
 * stage's stream can be restricted to one of n equal groups of compute units
 * (pipeline_partition_stream_create); a stage created on such a stream keeps its own
 * lanes on the same units.
 *
 * Conventions as in dapple_stage.h: 0 on success, a negative STAGE_E_* code otherwise,
 * message through stage_last_error(); pointers are DEVICE pointers unless they are
 * arrays of pointers or out-parameters, which are HOST memory; one handle is used by
 * one host thread at a time.
 */
#ifndef DAPPLE_PIPELINE_H
#define DAPPLE_PIPELINE_H

#include <stddef.h>
#include <stdint.h>

#include "dapple_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { PIPELINE_POLICY_A = 0, PIPELINE_POLICY_B = 1 };

/* K_i for i < S (section V-C): policy A min(S - i, D), policy B min(2(S - i) - 1, D), never
 * above M nor below 1; D <= 0 means "memory holds all M".  Host only. */
int pipeline_warmup_depths(int S, int M, int policy, int D, int32_t* K_out);

/* The planner's estimate of one iteration (section IV-A, equations 1 and 2) with the AllReduce term
 * at zero: L = T_w + T_s + T_e, T_w = sum_{s<=Q} F_s, T_s = (M-1)(F_Q + B_Q), T_e = sum_{a<=Q} B_a
 * (the maximum of equation 1 without AllReduce; the pivot's own last backward counts into the
 * ending phase).  F, B: S forward / backward task times; Q: the pivot stage, or -1 for the rule of
 * section IV-B-1 (start at the last stage, move to an earlier stage s when (M-1)(F_s+B_s) exceeds
 * (M-1)(F_Q+B_Q) plus the work of the stages between).  Host only. */
int pipeline_pivot_stage(int S, int M, const double* F, const double* B);
int pipeline_latency_model(int S, int M, const double* F, const double* B, int Q, double* L_out);

/* A stream that may only use compute units [part*n/nparts, (part+1)*n/nparts) of the n the
 * device has (nparts = 1: all of them): one of nparts virtual devices.  Default priority.
 * Create the stage of that virtual device with this stream; destroy the stage first. */
int pipeline_partition_stream_create(int part, int nparts, void** hip_stream_out);
int pipeline_partition_stream_destroy(void* hip_stream);

typedef struct dapple_pipeline* pipeline_handle;

/* Bytes of the boundary buffer: an activation and a gradient of act_bytes for each of the
 * S - 1 boundaries and each of max_M micro-batches. */
size_t pipeline_boundary_bytes(int S, int max_M, size_t act_bytes);

/* stages[0..S): live stage handles, each on its own non-NULL stream, all with the same
 * boundary tensor of act_bytes (b*s*H elements of the stage dtype); only the first may have
 * the embedding block and only the last the MLM head.  boundary_dev: at least
 * pipeline_boundary_bytes, 256-byte aligned, owned by the caller.  The handle keeps the
 * stage handles, it does not own them. */
int pipeline_create(pipeline_handle* out, int S, const stage_handle* stages, void* boundary_dev,
                    size_t boundary_bytes, size_t act_bytes, int max_M);
int pipeline_destroy(pipeline_handle p);

/* One iteration of M micro-batches.  K[0..S): warm-up depth per stage (each within its stage's
 * max_slots; must not grow along the pipeline or the lists deadlock: STAGE_E_BAD_ORDER, nothing
 * enqueued); order: STAGE_ORDER_EARLY_BACKWARD, or STAGE_ORDER_GPIPE (every stage runs all
 * forwards, then all backwards; K ignored, max_slots >= M needed).
 * xs[m]: input of stage 0 ([b*s, H], or int32 ids with the embedding block); ys[m]: output of
 * the last stage ([b*s, H], or float loss[1] with the head); dys[m]: gradient of ys[m] (NULL array
 * with the head); auxs[m]: int32 targets (head only, else NULL array); dxs[m]: gradient of xs[m]
 * (NULL array with the embedding block).  Accumulators are NOT cleared (stage_zero_grads).
 * Enqueues and returns; pipeline_sync waits for every stage. */
int pipeline_run(pipeline_handle p, int M, const int32_t* K, int order, const void* const* xs,
                 const void* const* dys, const void* const* auxs, void* const* ys, void* const* dxs);
int pipeline_sync(pipeline_handle p);

/* Times of the last pipeline_run (after pipeline_sync), in milliseconds from its start, from the
 * HIP events around every task: start_ms / end_ms [2 * S * M], index (kind * S + stage) * M + m
 * with kind 0 = forward, 1 = backward. */
int pipeline_timeline(pipeline_handle p, double* start_ms, double* end_ms, int capacity);

#ifdef __cplusplus
}
#endif
#endif
