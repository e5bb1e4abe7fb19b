"""Plain CPU definition of the profiled performance model and of the parallelism search.

TEST INFRASTRUCTURE ONLY (see stage_oracle.py): only tests and the benchmark's reporting may
import this file; the product never does and shares no code with it.

Performance model (Model Profiler, "Throughput Profiling" and "Memory Profiling"): throughput and
memory are measured on a grid of input sizes and TP degrees and read off between grid points by
linear interpolation.  Readings taken where the text is silent:
  * throughput outside the profiled range keeps the value of the nearest grid point (a throughput
    curve flattens; a straight continuation could turn negative);
  * memory outside the profiled range continues the nearest segment's straight line (activation
    memory keeps growing with the input);
  * memory is profiled at two layer counts and is a straight line in the layer count through
    those two points;
  * a TP degree between two profiled degrees interpolates linearly between their two curves.

Item durations (Data-aware 3D Parallelism Optimizer, "Problem Formulation"; Online Microbatch
Scheduler, "Scheduling Optimization"): duration = computational load / throughput at the item's own
shape; for the LLM the attention and the linear operations have separate throughput models
("Throughput Profiling"), so their two quotients add.

Parallelism search (Algorithm 1, Eq. 1-5).  Readings: a module's FLOP count in the algorithm is
the data set's average FLOPs per item times the items of one microbatch; TP degrees are limited
to one node (Eq. 2) and PP degrees to the module's layer count inside the enumeration; layers per
stage E_l / E_pp may be fractional; enumeration order is encoder GPUs ascending, then encoder
(tp, pp) ascending, then LLM (tp, pp) ascending, then the microbatch count ascending, and only a
strictly smaller makespan replaces the incumbent.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple


# ----------------------------------------------------------------------------- interpolation
def interp(xs: Sequence[float], ys: Sequence[float], q: float, extrapolate: bool) -> float:
    """Piecewise-linear through (xs[k], ys[k]), xs strictly ascending."""
    n = len(xs)
    if n == 1:
        return float(ys[0])
    if q <= xs[0]:
        k = 0
        if not extrapolate:
            return float(ys[0])
    elif q >= xs[n - 1]:
        k = n - 2
        if not extrapolate:
            return float(ys[n - 1])
    else:
        k = 0
        while not (xs[k] <= q < xs[k + 1]):
            k += 1
    t = (q - xs[k]) / (xs[k + 1] - xs[k])
    return float(ys[k] + t * (ys[k + 1] - ys[k]))


def over_tp(tps: Sequence[int], values: Sequence[float], tp: float) -> float:
    """values[r] belongs to the profiled degree tps[r]; linear between, held outside."""
    return interp([float(t) for t in tps], values, float(tp), extrapolate=False)


def throughput(prof: Dict, x: float, tp: float) -> float:
    """E_thr(b, tp) or L_thr(s, tp): FLOP/s per GPU."""
    rows = [interp(prof["x"], prof["thr"][r], x, extrapolate=False) for r in range(len(prof["tp"]))]
    return over_tp(prof["tp"], rows, tp)


def line_in_layers(prof: Dict, at_lo: float, at_hi: float, layers: float) -> float:
    lo, hi = prof["layers_lo"], prof["layers_hi"]
    return at_lo + (layers - lo) * (at_hi - at_lo) / (hi - lo)


def model_state(prof: Dict, layers: float, tp: float) -> float:
    rows = [line_in_layers(prof, prof["model_state"][r][0], prof["model_state"][r][1], layers)
            for r in range(len(prof["tp"]))]
    return over_tp(prof["tp"], rows, tp)


def act_state(prof: Dict, layers: float, tp: float, x: float) -> float:
    rows = []
    for r in range(len(prof["tp"])):
        a_lo = interp(prof["x"], prof["act_state"][r][0], x, extrapolate=True)
        a_hi = interp(prof["x"], prof["act_state"][r][1], x, extrapolate=True)
        rows.append(line_in_layers(prof, a_lo, a_hi, layers))
    return over_tp(prof["tp"], rows, tp)


# ----------------------------------------------------------------------------- item durations
def item_durations(e_thr: Tuple[Sequence[float], Sequence[float]],
                   l_attn_thr: Tuple[Sequence[float], Sequence[float]],
                   l_lin_thr: Tuple[Sequence[float], Sequence[float]],
                   b: Sequence[float], s: Sequence[float], e_flop: Sequence[float],
                   l_lin_flop: Sequence[float], l_attn_flop: Sequence[float]) -> Tuple[List[float], List[float]]:
    """Per item: encoder duration e_flop / E_thr(b) and LLM duration
    l_lin_flop / L_lin_thr(s) + l_attn_flop / L_attn_thr(s).  A zero load costs zero time."""
    e_dur, l_dur = [], []
    for i in range(len(b)):
        e = 0.0 if e_flop[i] == 0 else e_flop[i] / interp(e_thr[0], e_thr[1], b[i], False)
        lin = 0.0 if l_lin_flop[i] == 0 else l_lin_flop[i] / interp(l_lin_thr[0], l_lin_thr[1], s[i], False)
        att = 0.0 if l_attn_flop[i] == 0 else l_attn_flop[i] / interp(l_attn_thr[0], l_attn_thr[1], s[i], False)
        e_dur.append(e)
        l_dur.append(lin + att)
    return e_dur, l_dur


# ----------------------------------------------------------------------------- Algorithm 1
def find_combs(gpus: int, n_gpu_node: int, max_pp: int) -> List[Tuple[int, int, int]]:
    """All (tp, pp, dp) with tp * pp * dp == gpus, tp within a node, pp within the layer count."""
    out = []
    for tp in range(1, min(gpus, n_gpu_node) + 1):
        if gpus % tp:
            continue
        rest = gpus // tp
        for pp in range(1, min(rest, max_pp) + 1):
            if rest % pp == 0:
                out.append((tp, pp, rest // pp))
    return out


def mem_e(enc: Dict, e_tp, e_pp, bsz, l_pp) -> float:
    """Eq. 4: the encoder's activations stay alive for the whole pipeline depth."""
    lay = enc["n_layers"] / e_pp
    return model_state(enc, lay, e_tp) + (e_pp + l_pp) * act_state(enc, lay, e_tp, bsz)


def mem_l(llm: Dict, l_tp, l_pp, seq_len) -> float:
    """Eq. 5."""
    lay = llm["n_layers"] / l_pp
    return model_state(llm, lay, l_tp) + l_pp * act_state(llm, lay, l_tp, seq_len)


def makespan(n_mb: int, e_pp: int, l_pp: int, e_dur: float, l_dur: float) -> float:
    """Eq. 1."""
    return (n_mb + e_pp + l_pp - 1) * max(e_dur, l_dur)


def evaluate(enc: Dict, llm: Dict, theta: Sequence[int], m_gpu: float, gbs: int, mean_bsz: float,
             mean_seq_len: float) -> Optional[float]:
    """Makespan of one configuration, or None when it does not fit in memory (Phase 2's body)."""
    e_tp, e_pp, e_dp, l_tp, l_pp, l_dp, i = theta
    t_bsz = mean_bsz * gbs / (i * e_dp)
    t_seq = mean_seq_len * gbs / (i * l_dp)
    if mem_e(enc, e_tp, e_pp, t_bsz, l_pp) > m_gpu or mem_l(llm, l_tp, l_pp, t_seq) > m_gpu:
        return None
    e_flop = enc["flop_per_item"] * gbs / (i * e_dp)
    l_flop = llm["flop_per_item"] * gbs / (i * l_dp)
    e_dur = e_flop / (throughput(enc, t_bsz, e_tp) * e_tp * e_pp)
    l_dur = l_flop / (throughput(llm, t_seq, l_tp) * l_tp * l_pp)
    return makespan(i, e_pp, l_pp, e_dur, l_dur)


def optimize(enc: Dict, llm: Dict, n_gpus: int, n_gpu_node: int, m_gpu: float, gbs: int,
             mean_bsz: float, mean_seq_len: float) -> Tuple[Optional[Tuple[int, ...]], float]:
    """Algorithm 1: (theta*, min_T); theta* = (E_tp, E_pp, E_dp, L_tp, L_pp, L_dp, N_mb)."""
    configs = []
    for e_gpus in range(1, n_gpus):                                   # Phase 1
        l_gpus = n_gpus - e_gpus
        for ec in find_combs(e_gpus, n_gpu_node, int(enc["n_layers"])):
            for lc in find_combs(l_gpus, n_gpu_node, int(llm["n_layers"])):
                configs.append(ec + lc)
    min_t, best = math.inf, None
    for cfg in configs:                                               # Phase 2
        l_dp = cfg[5]
        for i in range(1, gbs // l_dp + 1):
            t = evaluate(enc, llm, cfg + (i,), m_gpu, gbs, mean_bsz, mean_seq_len)
            if t is not None and t < min_t:
                min_t, best = t, cfg + (i,)
    return best, min_t
