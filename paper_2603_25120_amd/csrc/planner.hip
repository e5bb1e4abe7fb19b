// Profiled performance model and the data-aware parallelism search (host code, no GPU work).
//
// Model Profiler ("Throughput Profiling", "Memory Profiling"): measured grids, linear
// interpolation in between.  Throughput is held constant outside the profiled range, memory is
// continued along its end segment; memory is a straight line in the layer count through the two
// profiled layer counts; TP degrees between two profiled ones blend their two curves linearly.
//
// Parallelism search: Algorithm 1 with Eq. 1 (makespan), Eq. 2-3 (TP inside a node, every GPU
// used), Eq. 4-5 (memory of the encoder and of the LLM at the mean microbatch shape).
#include <algorithm>
#include <atomic>
#include <cmath>
#include <limits>
#include <thread>
#include <vector>

#include "../../include/mllm_stage.h"

namespace mllm_detail { void set_last_error(const char* msg); }

namespace {

mllm_status_t pfail(mllm_status_t st, const char* msg) {
  mllm_detail::set_last_error(msg);
  return st;
}

// Segment [k, k+1] of an ascending grid that holds q (end segments also serve the outside).
int segment_of(const double* x, int n, double q) {
  int lo = 0, hi = n - 1;              // invariant: x[lo] <= q < x[hi] once q is inside
  if (q <= x[0]) return 0;
  if (q >= x[n - 1]) return n - 2;
  while (hi - lo > 1) {
    const int mid = (lo + hi) / 2;
    if (x[mid] <= q) lo = mid; else hi = mid;
  }
  return lo;
}

double pw_linear(const double* x, const double* y, int n, double q, bool extrapolate) {
  if (n == 1) return y[0];
  if (!extrapolate) {
    if (q <= x[0]) return y[0];
    if (q >= x[n - 1]) return y[n - 1];
  }
  const int k = segment_of(x, n, q);
  const double t = (q - x[k]) / (x[k + 1] - x[k]);
  return y[k] + t * (y[k + 1] - y[k]);
}

mllm_status_t check_curve(const mllm_curve_t* c, bool positive) {
  if (!c || !c->x || !c->y) return pfail(MLLM_ERR_NULL, "curve or its arrays are NULL");
  if (c->n < 1) return pfail(MLLM_ERR_SHAPE, "a curve needs at least one grid point");
  for (int k = 0; k < c->n; k++) {
    if (!std::isfinite(c->x[k]) || !std::isfinite(c->y[k])) return pfail(MLLM_ERR_SHAPE, "curve values must be finite");
    if (k > 0 && !(c->x[k] > c->x[k - 1])) return pfail(MLLM_ERR_SHAPE, "curve grid must be strictly ascending");
    if (positive && !(c->y[k] > 0.0)) return pfail(MLLM_ERR_SHAPE, "throughput values must be positive");
  }
  return MLLM_OK;
}

mllm_status_t check_profile(const mllm_module_profile_t* p) {
  if (!p || !p->tp || !p->x || !p->thr || !p->model_state || !p->act_state)
    return pfail(MLLM_ERR_NULL, "module profile or one of its tables is NULL");
  if (p->n_tp < 1 || p->n_x < 1 || p->n_layers < 1) return pfail(MLLM_ERR_SHAPE, "module profile: empty grid or no layers");
  if (!(p->layers_lo < p->layers_hi)) return pfail(MLLM_ERR_SHAPE, "module profile: need layers_lo < layers_hi");
  for (int r = 0; r < p->n_tp; r++)
    if (p->tp[r] < 1 || (r > 0 && p->tp[r] <= p->tp[r - 1])) return pfail(MLLM_ERR_SHAPE, "module profile: TP degrees must be positive and ascending");
  for (int k = 0; k < p->n_x; k++)
    if (!std::isfinite(p->x[k]) || (k > 0 && !(p->x[k] > p->x[k - 1]))) return pfail(MLLM_ERR_SHAPE, "module profile: input grid must be strictly ascending");
  for (int64_t k = 0; k < (int64_t)p->n_tp * p->n_x; k++)
    if (!(p->thr[k] > 0.0) || !std::isfinite(p->thr[k])) return pfail(MLLM_ERR_SHAPE, "module profile: throughput must be positive");
  if (!(p->flop_per_item >= 0.0)) return pfail(MLLM_ERR_SHAPE, "module profile: flop_per_item must be non-negative");
  return MLLM_OK;
}

// Where a TP degree falls among the profiled ones: value = v[k] + t * (v[k+1] - v[k]), or v[k]
// alone when single is set (a one-row table, or a degree outside the profiled range).
struct TpPos { int k; double t; bool single; };

TpPos locate_tp(const mllm_module_profile_t& p, double tp) {
  const int n = p.n_tp;
  if (n == 1 || tp <= p.tp[0]) return {0, 0.0, true};
  if (tp >= p.tp[n - 1]) return {n - 1, 0.0, true};
  int k = 0;
  while (!(p.tp[k] <= tp && tp < p.tp[k + 1])) k++;
  return {k, (tp - p.tp[k]) / (double)(p.tp[k + 1] - p.tp[k]), false};
}

template <class RowFn>
double blend_tp(const TpPos& w, RowFn row) {
  const double v0 = row(w.k);
  if (w.single) return v0;
  return v0 + w.t * (row(w.k + 1) - v0);
}

double thr_at(const mllm_module_profile_t& p, double x, double tp) {
  return blend_tp(locate_tp(p, tp), [&](int r) { return pw_linear(p.x, p.thr + (int64_t)r * p.n_x, p.n_x, x, false); });
}

double along_layers(const mllm_module_profile_t& p, double at_lo, double at_hi, double layers) {
  return at_lo + (layers - p.layers_lo) * (at_hi - at_lo) / (p.layers_hi - p.layers_lo);
}

double model_state_at(const mllm_module_profile_t& p, double layers, double tp) {
  return blend_tp(locate_tp(p, tp), [&](int r) {
    return along_layers(p, p.model_state[2 * r], p.model_state[2 * r + 1], layers);
  });
}

double act_state_at(const mllm_module_profile_t& p, double layers, double tp, double x) {
  return blend_tp(locate_tp(p, tp), [&](int r) {
    const double* base = p.act_state + (int64_t)r * 2 * p.n_x;
    return along_layers(p, pw_linear(p.x, base, p.n_x, x, true), pw_linear(p.x, base + p.n_x, p.n_x, x, true), layers);
  });
}

// The two halves of one pass of Phase 2's inner loop.  Each depends on its own module's degrees
// and on the microbatch count only (the encoder's memory also on L_pp, added by the caller), so
// the search computes them once per (degrees, count) and combines them per pair of modules.
struct EncSide { double dur, model_state, act; };
struct LlmSide { double dur, mem; };

EncSide enc_side(const mllm_module_profile_t& enc, double e_tp, double e_pp, double e_dp, double n_mb,
                 int32_t gbs, double mean_bsz) {
  const double t_bsz = mean_bsz * gbs / (n_mb * e_dp);
  const double layers = enc.n_layers / e_pp;
  EncSide r;
  r.model_state = model_state_at(enc, layers, e_tp);
  r.act = act_state_at(enc, layers, e_tp, t_bsz);
  const double flop = enc.flop_per_item * gbs / (n_mb * e_dp);
  r.dur = flop / (thr_at(enc, t_bsz, e_tp) * e_tp * e_pp);
  return r;
}

LlmSide llm_side(const mllm_module_profile_t& llm, double l_tp, double l_pp, double l_dp, double n_mb,
                 int32_t gbs, double mean_seq_len) {
  const double t_seq = mean_seq_len * gbs / (n_mb * l_dp);
  const double layers = llm.n_layers / l_pp;
  LlmSide r;
  r.mem = model_state_at(llm, layers, l_tp) + l_pp * act_state_at(llm, layers, l_tp, t_seq);   // Eq. 5
  const double flop = llm.flop_per_item * gbs / (n_mb * l_dp);
  r.dur = flop / (thr_at(llm, t_seq, l_tp) * l_tp * l_pp);
  return r;
}

struct Eval { double makespan, e_mem, l_mem; bool feasible; };

Eval combine(const EncSide& e, const LlmSide& l, double e_pp, double l_pp, double n_mb, double m_gpu) {
  Eval r;
  r.e_mem = e.model_state + (e_pp + l_pp) * e.act;                                            // Eq. 4
  r.l_mem = l.mem;
  r.feasible = !(r.e_mem > m_gpu) && !(r.l_mem > m_gpu);
  r.makespan = (n_mb + e_pp + l_pp - 1.0) * (e.dur > l.dur ? e.dur : l.dur);                   // Eq. 1
  return r;
}

Eval evaluate(const mllm_module_profile_t& enc, const mllm_module_profile_t& llm, const int32_t* th,
              double m_gpu, int32_t gbs, double mean_bsz, double mean_seq_len) {
  return combine(enc_side(enc, th[0], th[1], th[2], th[6], gbs, mean_bsz),
                 llm_side(llm, th[3], th[4], th[5], th[6], gbs, mean_seq_len), th[1], th[4], th[6], m_gpu);
}

struct Triple { int32_t tp, pp, dp; };

std::vector<Triple> combs(int32_t gpus, int32_t n_gpu_node, int32_t max_pp) {
  std::vector<Triple> out;
  for (int32_t tp = 1; tp <= gpus && tp <= n_gpu_node; tp++) {
    if (gpus % tp) continue;
    const int32_t rest = gpus / tp;
    for (int32_t pp = 1; pp <= rest && pp <= max_pp; pp++)
      if (rest % pp == 0) out.push_back({tp, pp, rest / pp});
  }
  return out;
}

struct Best { double t = std::numeric_limits<double>::infinity(); int32_t th[7] = {0, 0, 0, 0, 0, 0, 0}; bool found = false; };

// Phase 2 for one split (E_gpus, L_gpus), in the algorithm's order: encoder degrees, LLM degrees,
// microbatch count; a strictly smaller makespan replaces the incumbent.
Best search_split(const mllm_module_profile_t& enc, const mllm_module_profile_t& llm, int32_t e_gpus, int32_t l_gpus,
                  int32_t n_gpu_node, double m_gpu, int32_t gbs, double mean_bsz, double mean_seq_len) {
  Best best;
  const std::vector<Triple> ec = combs(e_gpus, n_gpu_node, enc.n_layers);
  const std::vector<Triple> lc = combs(l_gpus, n_gpu_node, llm.n_layers);
  if (ec.empty() || lc.empty()) return best;
  int32_t i_max = 0;
  std::vector<std::vector<LlmSide>> ls(lc.size());
  for (size_t b = 0; b < lc.size(); b++) {
    const int32_t n_max = gbs / lc[b].dp;
    i_max = std::max(i_max, n_max);
    ls[b].resize(n_max);
    for (int32_t i = 1; i <= n_max; i++) ls[b][i - 1] = llm_side(llm, lc[b].tp, lc[b].pp, lc[b].dp, i, gbs, mean_seq_len);
  }
  std::vector<EncSide> es(i_max);
  for (const Triple& e : ec) {
    for (int32_t i = 1; i <= i_max; i++) es[i - 1] = enc_side(enc, e.tp, e.pp, e.dp, i, gbs, mean_bsz);
    for (size_t b = 0; b < lc.size(); b++) {
      const Triple& l = lc[b];
      const int32_t n_max = gbs / l.dp;
      for (int32_t i = 1; i <= n_max; i++) {
        const Eval r = combine(es[i - 1], ls[b][i - 1], e.pp, l.pp, i, m_gpu);
        if (r.feasible && r.makespan < best.t) {
          best.t = r.makespan;
          const int32_t th[7] = {e.tp, e.pp, e.dp, l.tp, l.pp, l.dp, i};
          for (int k = 0; k < 7; k++) best.th[k] = th[k];
          best.found = true;
        }
      }
    }
  }
  return best;
}

}  // namespace

extern "C" {

mllm_status_t mllm_interp(const mllm_curve_t* curve, int64_t nq, const double* q, int32_t extrapolate, double* out) {
  if (mllm_status_t st = check_curve(curve, false)) return st;
  if (nq < 0) return pfail(MLLM_ERR_SHAPE, "nq must be non-negative");
  if (nq > 0 && (!q || !out)) return pfail(MLLM_ERR_NULL, "q or out is NULL");
  for (int64_t j = 0; j < nq; j++) out[j] = pw_linear(curve->x, curve->y, curve->n, q[j], extrapolate != 0);
  return MLLM_OK;
}

mllm_status_t mllm_item_durations(int64_t n_items, const double* b, const double* s, const double* e_flop,
                                  const double* l_lin_flop, const double* l_attn_flop, const mllm_curve_t* e_thr,
                                  const mllm_curve_t* l_lin_thr, const mllm_curve_t* l_attn_thr,
                                  double* e_dur_out, double* l_dur_out) {
  if (mllm_status_t st = check_curve(e_thr, true)) return st;
  if (mllm_status_t st = check_curve(l_lin_thr, true)) return st;
  if (mllm_status_t st = check_curve(l_attn_thr, true)) return st;
  if (n_items < 0) return pfail(MLLM_ERR_SHAPE, "n_items must be non-negative");
  if (n_items > 0 && (!b || !s || !e_flop || !l_lin_flop || !l_attn_flop || !e_dur_out || !l_dur_out))
    return pfail(MLLM_ERR_NULL, "an item array is NULL");
  for (int64_t i = 0; i < n_items; i++)
    if (!(e_flop[i] >= 0.0) || !(l_lin_flop[i] >= 0.0) || !(l_attn_flop[i] >= 0.0) || !std::isfinite(b[i]) || !std::isfinite(s[i]))
      return pfail(MLLM_ERR_SHAPE, "item loads must be non-negative and shapes finite");
  for (int64_t i = 0; i < n_items; i++) {
    e_dur_out[i] = e_flop[i] > 0.0 ? e_flop[i] / pw_linear(e_thr->x, e_thr->y, e_thr->n, b[i], false) : 0.0;
    const double lin = l_lin_flop[i] > 0.0 ? l_lin_flop[i] / pw_linear(l_lin_thr->x, l_lin_thr->y, l_lin_thr->n, s[i], false) : 0.0;
    const double att = l_attn_flop[i] > 0.0 ? l_attn_flop[i] / pw_linear(l_attn_thr->x, l_attn_thr->y, l_attn_thr->n, s[i], false) : 0.0;
    l_dur_out[i] = lin + att;
  }
  return MLLM_OK;
}

mllm_status_t mllm_find_combs(int32_t gpus, int32_t n_gpu_node, int32_t max_pp, int64_t capacity,
                              int32_t* triples_out, int64_t* count_out) {
  if (!count_out) return pfail(MLLM_ERR_NULL, "count_out is NULL");
  if (gpus < 1 || n_gpu_node < 1 || max_pp < 1 || capacity < 0) return pfail(MLLM_ERR_SHAPE, "gpus, n_gpu_node and max_pp must be >= 1");
  if (capacity > 0 && !triples_out) return pfail(MLLM_ERR_NULL, "triples_out is NULL");
  const std::vector<Triple> c = combs(gpus, n_gpu_node, max_pp);
  *count_out = (int64_t)c.size();
  for (int64_t k = 0; k < (int64_t)c.size() && k < capacity; k++) {
    triples_out[3 * k] = c[k].tp; triples_out[3 * k + 1] = c[k].pp; triples_out[3 * k + 2] = c[k].dp;
  }
  return MLLM_OK;
}

mllm_status_t mllm_evaluate_parallelism(const mllm_module_profile_t* enc, const mllm_module_profile_t* llm,
                                        const int32_t theta[7], double m_gpu, int32_t gbs, double mean_bsz,
                                        double mean_seq_len, double* makespan_out, double* e_mem_out,
                                        double* l_mem_out, int32_t* feasible_out) {
  if (mllm_status_t st = check_profile(enc)) return st;
  if (mllm_status_t st = check_profile(llm)) return st;
  if (!theta) return pfail(MLLM_ERR_NULL, "theta is NULL");
  for (int k = 0; k < 7; k++) if (theta[k] < 1) return pfail(MLLM_ERR_SHAPE, "every entry of theta must be >= 1");
  if (gbs < 1 || !(mean_bsz >= 0.0) || !(mean_seq_len >= 0.0)) return pfail(MLLM_ERR_SHAPE, "need gbs >= 1 and non-negative means");
  const Eval r = evaluate(*enc, *llm, theta, m_gpu, gbs, mean_bsz, mean_seq_len);
  if (makespan_out) *makespan_out = r.makespan;
  if (e_mem_out) *e_mem_out = r.e_mem;
  if (l_mem_out) *l_mem_out = r.l_mem;
  if (feasible_out) *feasible_out = r.feasible ? 1 : 0;
  return MLLM_OK;
}

mllm_status_t mllm_optimize_parallelism(const mllm_module_profile_t* enc, const mllm_module_profile_t* llm,
                                        int32_t n_gpus, int32_t n_gpu_node, double m_gpu, int32_t gbs,
                                        double mean_bsz, double mean_seq_len, int32_t theta_out[7],
                                        double* min_t_out, int32_t* found_out) {
  if (mllm_status_t st = check_profile(enc)) return st;
  if (mllm_status_t st = check_profile(llm)) return st;
  if (!theta_out || !min_t_out || !found_out) return pfail(MLLM_ERR_NULL, "an output pointer is NULL");
  if (n_gpus < 2 || n_gpu_node < 1 || gbs < 1) return pfail(MLLM_ERR_SHAPE, "need n_gpus >= 2 (one per module), n_gpu_node >= 1, gbs >= 1");
  if (!(mean_bsz >= 0.0) || !(mean_seq_len >= 0.0)) return pfail(MLLM_ERR_SHAPE, "means must be non-negative");
  // Every split of the GPUs is searched on its own (worker threads take splits in turn); the
  // per-split winners are then compared in the order of the sequential algorithm, so the result
  // does not depend on the number of threads.
  std::vector<Best> per_split(n_gpus);
  const unsigned hw = std::thread::hardware_concurrency();
  const int n_threads = (int)std::min<unsigned>(std::max(1u, hw), std::min<unsigned>(16u, (unsigned)(n_gpus - 1)));
  std::atomic<int32_t> next(1);
  auto work = [&]() {
    for (int32_t e_gpus = next.fetch_add(1); e_gpus < n_gpus; e_gpus = next.fetch_add(1))
      per_split[e_gpus] = search_split(*enc, *llm, e_gpus, n_gpus - e_gpus, n_gpu_node, m_gpu, gbs, mean_bsz, mean_seq_len);
  };
  if (n_threads <= 1) {
    work();
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < n_threads; t++) pool.emplace_back(work);
    for (std::thread& t : pool) t.join();
  }
  double min_t = std::numeric_limits<double>::infinity();
  int32_t best[7] = {0, 0, 0, 0, 0, 0, 0};
  bool found = false;
  for (int32_t e_gpus = 1; e_gpus < n_gpus; e_gpus++) {
    const Best& b = per_split[e_gpus];
    if (b.found && b.t < min_t) {
      min_t = b.t;
      for (int k = 0; k < 7; k++) best[k] = b.th[k];
      found = true;
    }
  }
  for (int k = 0; k < 7; k++) theta_out[k] = best[k];
  *min_t_out = min_t;
  *found_out = found ? 1 : 0;
  return MLLM_OK;
}

}  // extern "C"
