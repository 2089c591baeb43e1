/*
 * mux_plan.h -- C ABI of the task-fusion planner (paper section 3.3): which of the co-located fine-tuning tasks
 * are batched in space into one hybrid task (one call of the multiplexed layer per projection) and which hybrid
 * tasks follow each other in time.  Host code only: no device memory, no stream, nothing is launched.
 *
 * Conventions as in mux.h: plain C, a mux_status (or a value) comes back, mux_last_error() holds the text of the
 * last failure.  Every pointer is host memory owned by the caller; the library keeps none of them after the call.
 * Latencies carry whatever unit the profiles carry (the benchmark writes milliseconds).
 */
#ifndef MUX_PLAN_H_
#define MUX_PLAN_H_

#include <stddef.h>
#include <stdint.h>

#include "mux.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Profile of one operator over the token count (section 5, offline profiling): n_points >= 1 samples, tokens
 * strictly increasing and positive.  Between two samples the curve is linear; below the first sample it keeps the
 * first value; above the last it continues the last segment (with a single sample: proportional to the tokens). */
typedef struct {
  int32_t n_points;
  const int64_t* tokens;
  const double* value;
} mux_profile_curve;

/* One pipeline stage of Eq. 3: its BaseOps with their latency t_o(x), its fused adapter groups with the latency
 * t_a(x) and the GPU utilisation u_a(x) in (0, 1] of one member alone on x tokens, and the number of GPUs N_g the
 * BaseOps are sharded over. */
typedef struct {
  int32_t n_gpus;
  int32_t n_baseops;
  const mux_profile_curve* baseop_latency;   /* n_baseops entries */
  int32_t n_adapters;
  const mux_profile_curve* adapter_latency;  /* n_adapters entries */
  const mux_profile_curve* adapter_util;     /* n_adapters entries */
} mux_stage_model;

/* The cost model of section 3.3: S = n_stages pipeline stages, C = n_microbatches micro-batches (both >= 1). */
typedef struct {
  int32_t n_stages;
  const mux_stage_model* stages;
  int32_t n_microbatches;
} mux_cost_model;

/* Eq. 3: latency of the hybrid task made of `n_tasks` tasks with tokens[k] tokens each, on stage `stage`:
 *   sum over the BaseOps of t_o(sum_k n_k) / N_g  +  sum over the adapter groups of
 *   max( sum_k u_a(n_k) t_a(n_k), max_k t_a(n_k) ).
 * Eq. 4: its end-to-end latency, 2 sum_{s < S} L^(s) + 2 C max_s L^(s).
 * Both write the value to *out; MUX_ERR_INVALID_ARG on a null pointer, a bad curve, n_tasks < 1 or a token count < 1. */
mux_status mux_plan_stage_latency(const mux_cost_model* model, int32_t stage, int32_t n_tasks, const int64_t* tokens,
                                  double* out);
mux_status mux_plan_htask_latency(const mux_cost_model* model, int32_t n_tasks, const int64_t* tokens, double* out);

/* Eq. 6: the tasks are ordered by ascending token count (equal counts keep their given order) and cut into
 * consecutive hybrid tasks so that  L(first hybrid task) + sum over the others of L(hybrid task) / S  is minimal,
 * over every number of hybrid tasks from 1 to max_htasks (0: up to n_tasks).
 *   order[n_tasks]         out: task indices in the planner's order
 *   htask_begin[n_tasks+1] out: hybrid task h holds order[htask_begin[h]] .. order[htask_begin[h+1] - 1]
 *   n_htasks               out
 *   latency                out: the minimum (F* of Eq. 6)
 * Among equal minima the plan with the fewest hybrid tasks is returned.  Time O(M^2 (S + M)) as in the paper
 * (the end-to-end latencies of all M (M + 1) / 2 candidate hybrid tasks are computed once). */
mux_status mux_plan_fusion(const mux_cost_model* model, int32_t n_tasks, const int64_t* tokens, int32_t max_htasks,
                           int32_t* order, int32_t* htask_begin, int32_t* n_htasks, double* latency);

#ifdef __cplusplus
}
#endif
#endif /* MUX_PLAN_H_ */
