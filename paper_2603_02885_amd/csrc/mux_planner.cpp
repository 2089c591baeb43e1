// Task-fusion planner (section 3.3): cost model of a hybrid task (Eq. 3, Eq. 4) and the dynamic programme that
// cuts the token-sorted tasks into hybrid tasks (Eq. 6).  Host code, double precision.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <string>
#include <vector>

#include "mux_internal.h"
#include "mux_plan.h"

namespace {

using mux::fail;

bool curve_ok(const mux_profile_curve& c) {
  if (c.n_points < 1 || !c.tokens || !c.value) return false;
  for (int i = 0; i < c.n_points; ++i) {
    if (c.tokens[i] < 1 || !std::isfinite(c.value[i])) return false;
    if (i > 0 && c.tokens[i] <= c.tokens[i - 1]) return false;
  }
  return true;
}

mux_status check_model(const char* fn, const mux_cost_model* m) {
  if (!m || !m->stages || m->n_stages < 1 || m->n_microbatches < 1)
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": the model needs at least one stage and one micro-batch");
  for (int s = 0; s < m->n_stages; ++s) {
    const mux_stage_model& st = m->stages[s];
    if (st.n_gpus < 1 || st.n_baseops < 0 || st.n_adapters < 0 || (st.n_baseops > 0 && !st.baseop_latency) ||
        (st.n_adapters > 0 && (!st.adapter_latency || !st.adapter_util)))
      return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad stage");
    for (int o = 0; o < st.n_baseops; ++o)
      if (!curve_ok(st.baseop_latency[o])) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad BaseOp profile");
    for (int a = 0; a < st.n_adapters; ++a)
      if (!curve_ok(st.adapter_latency[a]) || !curve_ok(st.adapter_util[a]))
        return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad adapter profile");
  }
  return MUX_OK;
}

mux_status check_tokens(const char* fn, int32_t n_tasks, const int64_t* tokens) {
  if (n_tasks < 1 || !tokens) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": no tasks");
  for (int k = 0; k < n_tasks; ++k)
    if (tokens[k] < 1) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": a task without tokens cannot be planned");
  return MUX_OK;
}

double at(const mux_profile_curve& c, double x) {
  const int n = c.n_points;
  if (x <= (double)c.tokens[0]) return c.value[0];
  if (n == 1) return c.value[0] * (x / (double)c.tokens[0]);
  int hi = (int)(std::upper_bound(c.tokens, c.tokens + n, (int64_t)std::ceil(x) - 1) - c.tokens);   // first sample >= x
  if (hi >= n) hi = n - 1;                                                                           // beyond the last: its segment
  const double x0 = (double)c.tokens[hi - 1], x1 = (double)c.tokens[hi];
  return c.value[hi - 1] + (c.value[hi] - c.value[hi - 1]) * ((x - x0) / (x1 - x0));
}

// Eq. 3 for the tasks first..last-1 of `tok`
double stage_latency(const mux_stage_model& st, const int64_t* tok, int first, int last) {
  int64_t total = 0;
  for (int k = first; k < last; ++k) total += tok[k];
  double base = 0.0;
  for (int o = 0; o < st.n_baseops; ++o) base += at(st.baseop_latency[o], (double)total) / (double)st.n_gpus;
  double adapters = 0.0;
  for (int a = 0; a < st.n_adapters; ++a) {
    double weighted = 0.0, slowest = 0.0;
    for (int k = first; k < last; ++k) {
      const double lat = at(st.adapter_latency[a], (double)tok[k]);
      weighted += at(st.adapter_util[a], (double)tok[k]) * lat;
      slowest = std::max(slowest, lat);
    }
    adapters += std::max(weighted, slowest);
  }
  return base + adapters;
}

// Eq. 4
double htask_latency(const mux_cost_model& m, const int64_t* tok, int first, int last) {
  double warm = 0.0, slowest = 0.0;
  for (int s = 0; s < m.n_stages; ++s) {
    const double l = stage_latency(m.stages[s], tok, first, last);
    if (s + 1 < m.n_stages) warm += l;
    slowest = std::max(slowest, l);
  }
  return 2.0 * warm + 2.0 * (double)m.n_microbatches * slowest;
}

}  // namespace

extern "C" mux_status mux_plan_stage_latency(const mux_cost_model* model, int32_t stage, int32_t n_tasks,
                                             const int64_t* tokens, double* out) {
  static const char* fn = "mux_plan_stage_latency";
  if (mux_status s = check_model(fn, model)) return s;
  if (mux_status s = check_tokens(fn, n_tasks, tokens)) return s;
  if (!out || stage < 0 || stage >= model->n_stages) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad stage or null result");
  *out = stage_latency(model->stages[stage], tokens, 0, n_tasks);
  return MUX_OK;
}

extern "C" mux_status mux_plan_htask_latency(const mux_cost_model* model, int32_t n_tasks, const int64_t* tokens,
                                             double* out) {
  static const char* fn = "mux_plan_htask_latency";
  if (mux_status s = check_model(fn, model)) return s;
  if (mux_status s = check_tokens(fn, n_tasks, tokens)) return s;
  if (!out) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null result");
  *out = htask_latency(*model, tokens, 0, n_tasks);
  return MUX_OK;
}

extern "C" mux_status mux_plan_fusion(const mux_cost_model* model, int32_t n_tasks, const int64_t* tokens,
                                      int32_t max_htasks, int32_t* order, int32_t* htask_begin, int32_t* n_htasks,
                                      double* latency) {
  static const char* fn = "mux_plan_fusion";
  if (mux_status s = check_model(fn, model)) return s;
  if (mux_status s = check_tokens(fn, n_tasks, tokens)) return s;
  if (!order || !htask_begin || !n_htasks || !latency || max_htasks < 0)
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null result or negative limit");
  const int M = n_tasks, S = model->n_stages;
  const int limit = max_htasks == 0 ? M : std::min(M, (int)max_htasks);
  try {
    std::vector<int32_t> ord(M);
    std::iota(ord.begin(), ord.end(), 0);
    std::stable_sort(ord.begin(), ord.end(), [&](int32_t a, int32_t b) { return tokens[a] < tokens[b]; });
    std::vector<int64_t> tok(M);
    for (int i = 0; i < M; ++i) tok[i] = tokens[ord[i]];
    // end-to-end latency of every candidate hybrid task: the sorted tasks i .. m-1
    std::vector<double> L((size_t)(M + 1) * (M + 1), 0.0);
    for (int i = 0; i < M; ++i)
      for (int m = i + 1; m <= M; ++m) L[(size_t)i * (M + 1) + m] = htask_latency(*model, tok.data(), i, m);
    // F[n][m]: the first m tasks in n hybrid tasks; the first hybrid task counts in full, the others by their
    // average per-stage latency
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<double> F((size_t)(limit + 1) * (M + 1), inf);
    std::vector<int32_t> from((size_t)(limit + 1) * (M + 1), -1);
    for (int m = 1; m <= M; ++m) F[(size_t)1 * (M + 1) + m] = L[(size_t)0 * (M + 1) + m];
    for (int n = 2; n <= limit; ++n)
      for (int m = n; m <= M; ++m)
        for (int i = n - 1; i < m; ++i) {
          const double c = F[(size_t)(n - 1) * (M + 1) + i] + L[(size_t)i * (M + 1) + m] / (double)S;
          if (c < F[(size_t)n * (M + 1) + m]) { F[(size_t)n * (M + 1) + m] = c; from[(size_t)n * (M + 1) + m] = i; }
        }
    int best = 1;
    for (int n = 2; n <= limit; ++n)
      if (F[(size_t)n * (M + 1) + M] < F[(size_t)best * (M + 1) + M]) best = n;
    std::vector<int32_t> begins(best + 1);
    begins[best] = M;
    for (int n = best, m = M; n > 1; --n) { m = from[(size_t)n * (M + 1) + m]; begins[n - 1] = m; }
    begins[0] = 0;
    std::copy(ord.begin(), ord.end(), order);
    std::copy(begins.begin(), begins.end(), htask_begin);
    *n_htasks = best;
    *latency = F[(size_t)best * (M + 1) + M];
  } catch (const std::bad_alloc&) {
    return fail(MUX_ERR_HOST_NOMEM, std::string(fn) + ": out of host memory");
  }
  return MUX_OK;
}
