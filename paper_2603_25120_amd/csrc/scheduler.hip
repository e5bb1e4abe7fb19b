// Online microbatch scheduler (host code, no GPU work): partition the N items of a global batch
// into m buckets so that the largest stage time of any bucket is as small as possible.
//
// Online Microbatch Scheduler, "Problem Formulation": item i has an encoder-stage duration e[i]
// and an LLM-stage duration l[i]; bucket j has E_j = sum of e and L_j = sum of l over its items;
// minimise C_max = max(max_j E_j, max_j L_j).  "Scheduling Optimization": an exact search with a
// strict limit, and the longest-processing-time-first heuristic as the fallback.  The exact search
// here is a depth-first branch and bound bounded by a node count (deterministic, unlike a wall
// clock); it starts from the LPT solution, so giving up early still returns something at least as
// good as the fallback.
//
// Reading of the greedy rule (longest item first, into the least loaded bucket) for two stages: an
// item's duration is max(e, l), a bucket's load is max(E_j, L_j); ties go to the lower index.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <numeric>
#include <vector>

#include "../../include/mllm_stage.h"

namespace mllm_detail { void set_last_error(const char* msg); }

namespace {

mllm_status_t sfail(mllm_status_t st, const char* msg) {
  mllm_detail::set_last_error(msg);
  return st;
}

mllm_status_t check(int64_t n, const double* e, const double* l, int32_t m, const int32_t* out) {
  if (n < 0 || m <= 0) return sfail(MLLM_ERR_SHAPE, "need n_items >= 0 and n_buckets >= 1");
  if (n > 0 && (!e || !l || !out)) return sfail(MLLM_ERR_NULL, "e_dur, l_dur or bucket_out is NULL");
  for (int64_t i = 0; i < n; i++)
    if (!(e[i] >= 0.0) || !(l[i] >= 0.0)) return sfail(MLLM_ERR_SHAPE, "durations must be non-negative numbers");
  return MLLM_OK;
}

std::vector<int64_t> lpt_order(int64_t n, const double* e, const double* l) {
  std::vector<int64_t> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
    return std::max(e[a], l[a]) > std::max(e[b], l[b]);
  });
  return order;
}

void lpt_assign(int64_t n, const double* e, const double* l, int32_t m, const std::vector<int64_t>& order,
                int32_t* out) {
  std::vector<double> E(m, 0.0), L(m, 0.0);
  for (int64_t idx = 0; idx < n; idx++) {
    const int64_t i = order[idx];
    int32_t best = 0;
    double best_load = std::max(E[0], L[0]);
    for (int32_t j = 1; j < m; j++) {
      const double load = std::max(E[j], L[j]);
      if (load < best_load) { best_load = load; best = j; }
    }
    out[i] = best;
    E[best] += e[i];
    L[best] += l[i];
  }
}

// Objective with the items added in index order (the summation order of the definition).
double objective(int64_t n, const double* e, const double* l, int32_t m, const int32_t* assign) {
  std::vector<double> E(m, 0.0), L(m, 0.0);
  for (int64_t i = 0; i < n; i++) { E[assign[i]] += e[i]; L[assign[i]] += l[i]; }
  double c = 0.0;
  for (int32_t j = 0; j < m; j++) c = std::max(c, std::max(E[j], L[j]));
  return c;
}

struct Search {
  int64_t n; int32_t m;
  const double* e; const double* l;
  const std::vector<int64_t>& order;
  std::vector<double> E, L, rest_e, rest_l;   // rest_*[k] = sum over order[k..] of that duration
  std::vector<int32_t> cur, best;
  double best_c, floor_c;
  int64_t nodes, node_limit;
  bool exhausted = false;

  void run(int64_t k, double cmax_so_far, int32_t used) {
    if (exhausted || best_c <= floor_c) return;
    if (k == n) {
      if (cmax_so_far < best_c) { best_c = cmax_so_far; best = cur; }
      return;
    }
    if (++nodes > node_limit) { exhausted = true; return; }
    // the remaining work has to go somewhere: average load bound over both stages
    double sumE = rest_e[k], sumL = rest_l[k];
    for (int32_t j = 0; j < m; j++) { sumE += E[j]; sumL += L[j]; }
    if (std::max(cmax_so_far, std::max(sumE, sumL) / m) >= best_c) return;
    const int64_t i = order[k];
    // buckets never used so far are interchangeable: try only the first of them
    const int32_t limit = std::min<int32_t>(m, used + 1);
    for (int32_t j = 0; j < limit; j++) {
      const double c = std::max(cmax_so_far, std::max(E[j] + e[i], L[j] + l[i]));
      if (c >= best_c) continue;
      E[j] += e[i]; L[j] += l[i]; cur[i] = j;
      run(k + 1, c, std::max(used, j + 1));
      E[j] -= e[i]; L[j] -= l[i];
      if (exhausted) return;
    }
  }
};

}  // namespace

extern "C" {

mllm_status_t mllm_schedule_lpt(int64_t n_items, const double* e_dur, const double* l_dur, int32_t n_buckets,
                                int32_t* bucket_out) {
  mllm_status_t st = check(n_items, e_dur, l_dur, n_buckets, bucket_out);
  if (st != MLLM_OK) return st;
  lpt_assign(n_items, e_dur, l_dur, n_buckets, lpt_order(n_items, e_dur, l_dur), bucket_out);
  return MLLM_OK;
}

mllm_status_t mllm_schedule(int64_t n_items, const double* e_dur, const double* l_dur, int32_t n_buckets,
                            int64_t node_limit, int32_t* bucket_out, double* cmax_out, int32_t* optimal_out) {
  mllm_status_t st = check(n_items, e_dur, l_dur, n_buckets, bucket_out);
  if (st != MLLM_OK) return st;
  const std::vector<int64_t> order = lpt_order(n_items, e_dur, l_dur);
  lpt_assign(n_items, e_dur, l_dur, n_buckets, order, bucket_out);
  double best_c = objective(n_items, e_dur, l_dur, n_buckets, bucket_out);
  bool optimal = true;
  if (n_items > 0) {
    double floor_c = 0.0, se = 0.0, sl = 0.0;
    for (int64_t i = 0; i < n_items; i++) {
      floor_c = std::max(floor_c, std::max(e_dur[i], l_dur[i]));
      se += e_dur[i]; sl += l_dur[i];
    }
    floor_c = std::max(floor_c, std::max(se, sl) / n_buckets);
    Search s{n_items, n_buckets, e_dur, l_dur, order};
    s.E.assign(n_buckets, 0.0); s.L.assign(n_buckets, 0.0);
    s.rest_e.assign(n_items + 1, 0.0); s.rest_l.assign(n_items + 1, 0.0);
    for (int64_t k = n_items - 1; k >= 0; k--) {
      s.rest_e[k] = s.rest_e[k + 1] + e_dur[order[k]];
      s.rest_l[k] = s.rest_l[k + 1] + l_dur[order[k]];
    }
    s.cur.assign(n_items, 0);
    s.best.assign(bucket_out, bucket_out + n_items);
    s.best_c = best_c; s.floor_c = floor_c; s.nodes = 0; s.node_limit = std::max<int64_t>(node_limit, 0);
    s.run(0, 0.0, 0);
    optimal = !s.exhausted;
    if (s.best_c < best_c) {
      std::copy(s.best.begin(), s.best.end(), bucket_out);
      best_c = objective(n_items, e_dur, l_dur, n_buckets, bucket_out);
    }
  }
  if (cmax_out) *cmax_out = best_c;
  if (optimal_out) *optimal_out = optimal ? 1 : 0;
  return MLLM_OK;
}

}  // extern "C"
