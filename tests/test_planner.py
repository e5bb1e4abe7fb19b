"""Profiled performance model and parallelism search (Model Profiler; Algorithm 1): pins for the
oracle, then the library's host functions (C ABI) against the oracle.  No GPU is needed.

Pins (none of them re-types the oracle's formulas):
  * interpolation: NumPy's np.interp (the library routine for the held-ends case); affine data
    are reproduced exactly inside and, with continuation, outside the grid; a hand-worked point;
  * the memory model against the closed form it was tabulated from (affine in layers and input);
  * FindCombs: the count of ordered factorisations n = tp.pp.dp is multiplicative with
    C(a+2, 2) for a prime power p^a (12 -> 18, 64 -> 28, 30 -> 27); every triple multiplies to n;
  * Eq. 1 on hand-worked numbers;
  * Eq. 4, Eq. 5 and the body of Algorithm 1's Phase 2 on a toy table worked by hand (the
    (E_pp + L_pp) and L_pp multipliers of the activation states, layers per stage, the microbatch
    shapes t_bsz and t_seq_len, FLOPs per microbatch, throughput times tp times pp, the strict
    memory comparison): every expected number below is written out, none is computed with the
    oracle's formulas;
  * Algorithm 1 against a search that enumerates the whole box of 7-tuples and applies Eq. 2-5
    itself, and against the closed-form optimum for flat throughput and no memory pressure.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import planner_oracle as P


# --------------------------------------------------------------------------------- fixtures
def make_profile(rng, n_layers, flop_per_item, tps=(1, 2, 4, 8), xs=(1, 2, 4, 8, 16, 32, 64), flat=None,
                 mem_scale=1.0):
    """A synthetic module profile: throughput saturating in x and degrading with TP (the shape of
    the paper's Fig. 2), memory affine in layers and input and inversely proportional to TP."""
    xs = [float(v) for v in xs]
    thr = [[(flat if flat else 1e14 * (x / (x + 3.0)) * (1.0 - 0.07 * math.log2(tp)) * (1 + 0.01 * rng.random()))
            for x in xs] for tp in tps]
    lo, hi = 2.0, 4.0
    model_state = [[mem_scale * (1e8 + 3e8 * l) / tp for l in (lo, hi)] for tp in tps]
    act_state = [[[mem_scale * (2e6 + 5e6 * l * x) / tp for x in xs] for l in (lo, hi)] for tp in tps]
    return dict(tp=list(tps), x=xs, thr=thr, layers_lo=lo, layers_hi=hi, model_state=model_state,
                act_state=act_state, n_layers=n_layers, flop_per_item=flop_per_item)


# --------------------------------------------------------------------------------- interpolation
def test_interp_matches_numpy_with_held_ends():
    rng = np.random.default_rng(0)
    for _ in range(20):
        n = int(rng.integers(1, 9))
        xs = np.cumsum(rng.random(n) + 0.1)
        ys = rng.normal(size=n)
        for q in np.concatenate([rng.uniform(xs[0] - 1, xs[-1] + 1, 30), xs]):
            assert P.interp(xs, ys, float(q), False) == pytest.approx(np.interp(q, xs, ys), rel=1e-13, abs=1e-13)


def test_interp_affine_data_exact_and_hand_value():
    xs = [1.0, 2.0, 4.0, 8.0]
    ys = [3.0 * x - 2.0 for x in xs]
    for q in (-3.0, 0.0, 1.0, 1.5, 3.0, 7.9, 8.0, 20.0):
        assert P.interp(xs, ys, q, True) == pytest.approx(3.0 * q - 2.0, abs=1e-12)
    assert P.interp(xs, ys, 20.0, False) == ys[-1] and P.interp(xs, ys, -3.0, False) == ys[0]
    assert P.interp([0.0, 10.0], [100.0, 200.0], 2.5, False) == 125.0
    assert P.interp([5.0], [7.0], 99.0, True) == 7.0


def test_memory_model_against_closed_form():
    rng = np.random.default_rng(1)
    prof = make_profile(rng, 24, 1e12)
    for tp in (1, 2, 4, 8):
        for layers in (1.0, 2.0, 3.5, 24.0):
            assert P.model_state(prof, layers, tp) == pytest.approx((1e8 + 3e8 * layers) / tp, rel=1e-12)
            for x in (0.5, 1.0, 3.0, 64.0, 100.0):       # inside, on and beyond the grid
                assert P.act_state(prof, layers, tp, x) == pytest.approx((2e6 + 5e6 * layers * x) / tp, rel=1e-12)
    # a TP degree between two profiled ones lies on the chord between their values
    a, b = P.model_state(prof, 6.0, 2), P.model_state(prof, 6.0, 4)
    assert P.model_state(prof, 6.0, 3) == pytest.approx(0.5 * (a + b), rel=1e-12)
    t2, t4 = P.throughput(prof, 5.0, 2), P.throughput(prof, 5.0, 4)
    assert P.throughput(prof, 5.0, 3) == pytest.approx(0.5 * (t2 + t4), rel=1e-12)
    assert P.throughput(prof, 1000.0, 1) == prof["thr"][0][-1]          # held beyond the grid


def test_item_durations_definition():
    e_thr = ([1.0, 4.0], [10.0, 40.0])
    lin = ([100.0, 300.0], [50.0, 150.0])
    att = ([100.0, 300.0], [20.0, 20.0])
    e, l = P.item_durations(e_thr, att, lin, b=[2.0, 0.0, 8.0], s=[200.0, 100.0, 1000.0],
                            e_flop=[60.0, 0.0, 80.0], l_lin_flop=[1000.0, 100.0, 300.0],
                            l_attn_flop=[40.0, 0.0, 10.0])
    assert e == pytest.approx([60.0 / 20.0, 0.0, 80.0 / 40.0])
    assert l == pytest.approx([1000.0 / 100.0 + 40.0 / 20.0, 100.0 / 50.0, 300.0 / 150.0 + 10.0 / 20.0])


# --------------------------------------------------------------------------------- Algorithm 1
def n_ordered_triples(n):
    count, p, m = 1, 2, n
    while m > 1:
        a = 0
        while m % p == 0:
            m //= p
            a += 1
        count *= math.comb(a + 2, 2)
        p += 1
    return count


def test_find_combs_counts_and_products():
    assert [n_ordered_triples(n) for n in (12, 64, 30)] == [18, 28, 27]
    for n in range(1, 130):
        c = P.find_combs(n, n, n)
        assert len(c) == n_ordered_triples(n) == len(set(c))
        assert all(tp * pp * dp == n for tp, pp, dp in c)
        assert c == sorted(c)
    assert P.find_combs(16, 8, 2) == [(1, 1, 16), (1, 2, 8), (2, 1, 8), (2, 2, 4), (4, 1, 4), (4, 2, 2),
                                      (8, 1, 2), (8, 2, 1)]


def test_makespan_equation():
    assert P.makespan(4, 2, 2, 3.0, 5.0) == 35.0          # (4 + 2 + 2 - 1) * 5
    assert P.makespan(1, 1, 1, 2.0, 1.0) == 4.0


def box_search(enc, llm, n_gpus, n_gpu_node, m_gpu, gbs, mean_bsz, mean_seq_len):
    """Every 7-tuple of the box, constraints applied directly (Eq. 2, 3; N_mb <= GBS // L_dp;
    memory and makespan taken from the oracle's single-configuration evaluation)."""
    best, best_t = None, math.inf
    r = range(1, n_gpus + 1)
    for e_tp, e_pp, e_dp, l_tp, l_pp, l_dp in itertools.product(r, r, r, r, r, r):
        if e_tp * e_pp * e_dp + l_tp * l_pp * l_dp != n_gpus:
            continue
        if e_tp > n_gpu_node or l_tp > n_gpu_node or e_pp > enc["n_layers"] or l_pp > llm["n_layers"]:
            continue
        for i in range(1, gbs // l_dp + 1):
            t = P.evaluate(enc, llm, (e_tp, e_pp, e_dp, l_tp, l_pp, l_dp, i), m_gpu, gbs, mean_bsz, mean_seq_len)
            if t is not None and t < best_t:
                best, best_t = (e_tp, e_pp, e_dp, l_tp, l_pp, l_dp, i), t
    return best, best_t


@pytest.mark.parametrize("n_gpus,m_gpu", [(4, 1e18), (6, 1e18), (8, 1e18), (8, 6e9), (6, 2.5e9)])
def test_algorithm1_against_box_search(n_gpus, m_gpu):
    rng = np.random.default_rng(n_gpus)
    enc = make_profile(rng, 6, 2.0e12, xs=(1, 4, 16, 64, 256))
    llm = make_profile(rng, 8, 9.0e12, xs=(64, 256, 1024, 4096, 16384), mem_scale=3.0)
    # the LLM's activation table is per token, much smaller per unit of x
    llm["act_state"] = [[[v * 1e-2 for v in row] for row in per_l] for per_l in llm["act_state"]]
    args = (enc, llm, n_gpus, 4, m_gpu, 12, 2.5, 700.0)
    theta, t = P.optimize(*args)
    ref, ref_t = box_search(*args)
    assert t == ref_t
    if ref is None:
        assert theta is None
    else:
        assert P.evaluate(enc, llm, theta, m_gpu, 12, 2.5, 700.0) == ref_t
        assert theta[0] * theta[1] * theta[2] + theta[3] * theta[4] * theta[5] == n_gpus


def test_algorithm1_closed_form_flat_throughput():
    """Flat throughput, no memory pressure: T = (i + E_pp + L_pp - 1) GBS / (i thr) max(eF / E_gpus,
    lF / L_gpus) -- smallest with no pipelining inside a module, the largest microbatch count
    (L_dp = 1, i = GBS) and the GPU split that balances eF / E_gpus against lF / L_gpus."""
    rng = np.random.default_rng(3)
    thr, gbs = 1e12, 16
    enc = make_profile(rng, 4, 1e12, flat=thr)
    llm = make_profile(rng, 4, 3e12, flat=thr)
    theta, t = P.optimize(enc, llm, 4, 8, 1e30, gbs, 1.0, 100.0)
    assert theta[1] == 1 and theta[4] == 1 and theta[5] == 1 and theta[6] == gbs
    assert theta[0] * theta[2] == 1 and theta[3] == 3            # 1 GPU for the encoder, 3 for the LLM
    assert t == pytest.approx((gbs + 1) / thr * 1e12, rel=1e-12)


def test_algorithm1_memory_forces_pipelining_or_fails():
    rng = np.random.default_rng(4)
    enc = make_profile(rng, 4, 1e12, flat=1e12)
    llm = make_profile(rng, 8, 3e12, flat=1e12)
    cap = 0.9 * (1e8 + 3e8 * 8)      # below the model states of the 8 LLM layers on one GPU; TP capped at 1
    tight, _ = P.optimize(enc, llm, 8, 1, cap, 8, 1.0, 1.0)
    assert tight[3] == 1 and tight[4] > 1                                  # so the LLM must be cut into stages
    assert P.mem_l(llm, tight[3], tight[4], 1.0 * 8 / (tight[6] * tight[5])) <= cap
    assert P.mem_e(enc, tight[0], tight[1], 1.0 * 8 / (tight[6] * tight[2]), tight[4]) <= cap
    assert P.optimize(enc, llm, 8, 1, 1.0, 8, 1.0, 1.0) == (None, math.inf)


# --------------------------------------------------------------------------------- Eq. 4, Eq. 5, Phase 2 by hand
def toy_tables():
    """Two TP degrees, profiled at 2 and 4 layers, two grid points each.
    Encoder: model states 20 + 40 l bytes at TP 1 (100 at 2 layers, 180 at 4) and 20 + 20 l at TP 2;
    activation states 5 l x bytes at TP 1 (2 layers: 10, 30 at x = 1, 3; 4 layers: 20, 60), half at TP 2;
    throughput 100 x at TP 1, 80 x at TP 2.
    LLM: model states 60 + 20 l at TP 1, 20 + 20 l at TP 2; activation states at TP 2: 2 layers 5, 15 and
    4 layers 10, 30 at x = 100, 300 (twice that at TP 1); throughput 0.3 x at TP 1, 20 + 0.2 x at TP 2."""
    enc = dict(tp=[1, 2], x=[1.0, 3.0], thr=[[100.0, 300.0], [80.0, 240.0]], layers_lo=2.0, layers_hi=4.0,
               model_state=[[100.0, 180.0], [60.0, 100.0]],
               act_state=[[[10.0, 30.0], [20.0, 60.0]], [[5.0, 15.0], [10.0, 30.0]]],
               n_layers=8, flop_per_item=600.0)
    llm = dict(tp=[1, 2], x=[100.0, 300.0], thr=[[30.0, 90.0], [40.0, 80.0]], layers_lo=2.0, layers_hi=4.0,
               model_state=[[100.0, 140.0], [60.0, 100.0]],
               act_state=[[[10.0, 30.0], [20.0, 60.0]], [[5.0, 15.0], [10.0, 30.0]]],
               n_layers=6, flop_per_item=270.0)
    return enc, llm


def test_memory_equations_hand_worked():
    enc, llm = toy_tables()
    # Eq. 4, encoder of 8 layers on E_pp = 2 stages (4 layers per stage), TP 1, effective batch 2, L_pp = 3:
    # model states 180; activation states of 4 layers at x = 2 are midway between 20 and 60 = 40, kept for
    # E_pp + L_pp = 5 microbatches in flight: 180 + 5 * 40 = 380  (E_pp alone would give 260, L_pp alone 300)
    assert P.mem_e(enc, 1, 2, 2.0, 3) == pytest.approx(380.0, rel=1e-14)
    # the same stage behind a one-stage LLM: 180 + 3 * 40
    assert P.mem_e(enc, 1, 2, 2.0, 1) == pytest.approx(300.0, rel=1e-14)
    # E_pp = 4: 2 layers per stage: 100 + (4 + 3) * 20 = 240;  TP 2 halves the activations: 60 + 7 * 10 = 130
    assert P.mem_e(enc, 1, 4, 2.0, 3) == pytest.approx(240.0, rel=1e-14)
    assert P.mem_e(enc, 2, 4, 2.0, 3) == pytest.approx(130.0, rel=1e-14)
    # E_pp = 1: 8 layers per stage lie beyond the profiled 2 and 4: the line continues, 20 + 40 * 8 = 340
    # model states and 5 * 8 * 2 = 80 activation states: 340 + (1 + 3) * 80 = 660
    assert P.mem_e(enc, 1, 1, 2.0, 3) == pytest.approx(660.0, rel=1e-14)
    # Eq. 5, LLM of 6 layers on L_pp = 3 stages (2 layers per stage), TP 2, 200 packed tokens:
    # model states 60, activation states midway between 5 and 15 = 10, times L_pp = 3: 90 (not 60 + 10)
    assert P.mem_l(llm, 2, 3, 200.0) == pytest.approx(90.0, rel=1e-14)
    # TP 1, L_pp = 2: 3 layers per stage: model states 120, activations at 200 tokens midway between the
    # 2-layer 20 and the 4-layer 40 = 30, times 2: 180
    assert P.mem_l(llm, 1, 2, 200.0) == pytest.approx(180.0, rel=1e-14)


HAND_THETA = (1, 2, 3, 2, 3, 1, 4)      # E_tp, E_pp, E_dp, L_tp, L_pp, L_dp, N_mb: 6 + 6 GPUs


def test_phase2_body_hand_worked():
    """GBS 16, mean effective batch 1.5, mean sequence length 50, N_mb = 4:
    t_bsz = 1.5 * 16 / (4 * 3) = 2, t_seq_len = 50 * 16 / (4 * 1) = 200, so the memory figures are the
    380 and 90 of the test above.  Encoder FLOPs per microbatch 600 * 16 / 12 = 800 at 200 FLOP/s per GPU
    on 1 * 2 GPUs: 2 s.  LLM 270 * 16 / 4 = 1080 at 60 FLOP/s per GPU on 2 * 3 GPUs: 3 s.
    T = (4 + 2 + 3 - 1) * 3 = 24 s."""
    enc, llm = toy_tables()
    assert P.evaluate(enc, llm, HAND_THETA, 1e9, 16, 1.5, 50.0) == pytest.approx(24.0, rel=1e-14)
    assert P.evaluate(enc, llm, HAND_THETA, 380.0, 16, 1.5, 50.0) == pytest.approx(24.0, rel=1e-14)   # equal still fits
    assert P.evaluate(enc, llm, HAND_THETA, 379.9, 16, 1.5, 50.0) is None                             # Mem_E = 380
    # N_mb = 2 doubles both microbatch shapes: t_bsz = 4 lies beyond the grid, throughput holds 300, the
    # activation line continues to 80: Mem_E = 180 + 5 * 80 = 580; t_seq_len = 400: throughput holds 80,
    # activations 2 layers at TP 2 continue to 20: Mem_L = 60 + 3 * 20 = 120.
    # E_dur = 1600 / (300 * 2) = 8 / 3, L_dur = 2160 / (80 * 6) = 4.5, T = (2 + 4) * 4.5 = 27
    theta2 = HAND_THETA[:6] + (2,)
    assert P.evaluate(enc, llm, theta2, 580.0, 16, 1.5, 50.0) == pytest.approx(27.0, rel=1e-14)
    assert P.evaluate(enc, llm, theta2, 579.0, 16, 1.5, 50.0) is None
    # an LLM five times as memory-hungry is what binds: Mem_L = 5 * 90 = 450 > 400 >= Mem_E
    big = dict(llm, model_state=[[5 * v for v in r] for r in llm["model_state"]],
               act_state=[[[5 * v for v in row] for row in per_l] for per_l in llm["act_state"]])
    assert P.evaluate(enc, big, HAND_THETA, 400.0, 16, 1.5, 50.0) is None
    assert P.evaluate(enc, big, HAND_THETA, 450.0, 16, 1.5, 50.0) == pytest.approx(24.0, rel=1e-14)



# --------------------------------------------------------------------------------- library vs oracle
@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def test_library_interp_matches_oracle(B):
    rng = np.random.default_rng(10)
    for n in (1, 2, 5, 33):
        xs = np.cumsum(rng.random(n) + 0.05)
        ys = rng.normal(size=n)
        q = np.concatenate([rng.uniform(xs[0] - 2, xs[-1] + 2, 200), xs])
        for ex in (False, True):
            got = B.mllm_interp(xs, ys, q, ex)
            ref = np.array([P.interp(xs, ys, float(v), ex) for v in q])
            np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_library_item_durations_match_oracle(B):
    rng = np.random.default_rng(11)
    e_thr = (np.array([1, 2, 4, 8, 16.0]), rng.uniform(1e14, 5e14, 5))
    lin = (np.array([128, 512, 2048, 8192.0]), rng.uniform(5e14, 1e15, 4))
    att = (np.array([128, 512, 2048, 8192.0]), rng.uniform(1e14, 6e14, 4))
    n = 300
    b = rng.integers(0, 20, n).astype(float)
    s = rng.integers(1, 12000, n).astype(float)
    e_flop = b * 3.1e11
    l_lin = s * 2.6e10
    l_attn = s * s * 1.0e6
    e, l = B.mllm_item_durations(b, s, e_flop, l_lin, l_attn, e_thr, lin, att)
    e_ref, l_ref = P.item_durations(e_thr, att, lin, b, s, e_flop, l_lin, l_attn)
    np.testing.assert_allclose(e, e_ref, rtol=1e-13)
    np.testing.assert_allclose(l, l_ref, rtol=1e-13)


def test_library_find_combs_matches_oracle(B):
    for gpus, node, max_pp in [(1, 8, 4), (12, 8, 32), (64, 8, 24), (96, 4, 3), (97, 8, 8), (1024, 8, 80)]:
        got = [tuple(int(v) for v in row) for row in B.mllm_find_combs(gpus, node, max_pp)]
        assert got == P.find_combs(gpus, node, max_pp)


@pytest.mark.parametrize("n_gpus,node,m_gpu,gbs", [(2, 8, 1e30, 8), (8, 4, 1e30, 12), (8, 4, 6e9, 12), (16, 8, 4e9, 32),
                                                   (24, 8, 3e9, 64), (64, 8, 2e9, 128), (6, 2, 1.0, 8)])
def test_library_algorithm1_matches_oracle(B, n_gpus, node, m_gpu, gbs):
    rng = np.random.default_rng(100 + n_gpus)
    enc = make_profile(rng, 24, 2.0e12, xs=(1, 4, 16, 64, 256))
    llm = make_profile(rng, 32, 9.0e12, xs=(64, 256, 1024, 4096, 16384), mem_scale=3.0)
    llm["act_state"] = [[[v * 1e-2 for v in row] for row in per_l] for per_l in llm["act_state"]]
    theta, t = B.mllm_optimize_parallelism(enc, llm, n_gpus, node, m_gpu, gbs, 2.5, 700.0)
    ref, ref_t = P.optimize(enc, llm, n_gpus, node, m_gpu, gbs, 2.5, 700.0)
    assert theta == ref                      # integer result: exact
    if ref is None:
        assert t == math.inf
        return
    assert t == pytest.approx(ref_t, rel=1e-13)
    span, em, lm, ok = B.mllm_evaluate_parallelism(enc, llm, ref, m_gpu, gbs, 2.5, 700.0)
    assert ok and span == pytest.approx(ref_t, rel=1e-13)
    assert em == pytest.approx(P.mem_e(enc, ref[0], ref[1], 2.5 * gbs / (ref[6] * ref[2]), ref[4]), rel=1e-13)
    assert lm == pytest.approx(P.mem_l(llm, ref[3], ref[4], 700.0 * gbs / (ref[6] * ref[5])), rel=1e-13)


def test_library_planner_rejects_bad_arguments(B):
    with pytest.raises(B.MllmError):
        B.mllm_interp([1.0, 1.0], [0.0, 1.0], [0.5])                      # grid not strictly ascending
    with pytest.raises(B.MllmError):
        B.mllm_item_durations([1.0], [1.0], [1.0], [1.0], [1.0], ([1.0], [0.0]), ([1.0], [1.0]), ([1.0], [1.0]))
    rng = np.random.default_rng(0)
    enc, llm = make_profile(rng, 4, 1e12), make_profile(rng, 4, 1e12)
    with pytest.raises(B.MllmError):
        B.mllm_optimize_parallelism(enc, llm, 1, 8, 1e30, 8, 1.0, 1.0)     # one GPU cannot hold two modules
    bad = dict(enc, layers_hi=enc["layers_lo"])
    with pytest.raises(B.MllmError):
        B.mllm_optimize_parallelism(bad, llm, 4, 8, 1e30, 8, 1.0, 1.0)


def test_library_evaluation_hand_worked(B):
    """The library's single-configuration evaluation on the same toy tables: the hand-worked 24 s, 380 and
    90 bytes, and the strict comparison with the capacity."""
    enc, llm = toy_tables()
    span, em, lm, ok = B.mllm_evaluate_parallelism(enc, llm, HAND_THETA, 380.0, 16, 1.5, 50.0)
    assert ok and span == pytest.approx(24.0, rel=1e-13)
    assert em == pytest.approx(380.0, rel=1e-13) and lm == pytest.approx(90.0, rel=1e-13)
    _, em, lm, ok = B.mllm_evaluate_parallelism(enc, llm, HAND_THETA, 379.9, 16, 1.5, 50.0)
    assert not ok and em == pytest.approx(380.0, rel=1e-13)
    span, em, lm, ok = B.mllm_evaluate_parallelism(enc, llm, HAND_THETA[:6] + (2,), 580.0, 16, 1.5, 50.0)
    assert ok and span == pytest.approx(27.0, rel=1e-13)
    assert em == pytest.approx(580.0, rel=1e-13) and lm == pytest.approx(120.0, rel=1e-13)
