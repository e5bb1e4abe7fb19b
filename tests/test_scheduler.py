"""Online microbatch scheduler: pins for the oracle, then the library's scheduler (C ABI, host
only) against the oracle.  No GPU is needed.

Pins: the textbook worst case of LPT (Graham 1969, the source the paper cites for its fallback):
m = 3 identical machines and jobs 5,5,4,4,3,3,3 -- LPT gives makespan 11, the optimum is 9, the
ratio 4/3 - 1/(3m); brute force over all assignments on tiny instances; the bound
C_max >= max(sum e / m, sum l / m, largest item); invariants of the objective.
"""
import ctypes as C
import random

import numpy as np
import pytest

from oracle import scheduler_oracle as S


def test_objective_definition():
    e, l = [3.0, 1.0, 2.0], [1.0, 4.0, 1.0]
    assert S.bucket_times(e, l, [0, 1, 0], 2) == ([5.0, 1.0], [2.0, 4.0])
    assert S.c_max(e, l, [0, 1, 0], 2) == 5.0
    assert S.c_max(e, l, [0, 0, 0], 2) == 6.0      # everything in one bucket: max(sum e, sum l)


def test_lpt_textbook_worst_case():
    jobs = [5, 5, 4, 4, 3, 3, 3]
    zero = [0] * len(jobs)
    a = S.lpt(jobs, zero, 3)
    assert S.c_max(jobs, zero, a, 3) == 11
    opt, _ = S.brute_force(jobs, zero, 3)
    assert opt == 9
    assert 11 / 9 == pytest.approx(4 / 3 - 1 / 9)
    # the same jobs on the other stage give the same answer (the two stages are symmetric)
    assert S.c_max(zero, jobs, S.lpt(zero, jobs, 3), 3) == 11


def test_lpt_order_and_ties():
    # durations max(e,l) = 4, 4, 2, 1: items 0 and 1 tie (lower index first), buckets tie likewise
    e, l = [4, 1, 2, 1], [0, 4, 0, 0]
    assert S.lpt(e, l, 2) == [0, 1, 0, 1]


def test_brute_force_bounds_and_lpt_guarantee():
    rng = random.Random(5)
    for _ in range(40):
        n, m = rng.randint(1, 7), rng.randint(1, 3)
        e = [rng.randint(0, 9) for _ in range(n)]
        l = [rng.randint(0, 9) for _ in range(n)]
        opt, assign = S.brute_force(e, l, m)
        assert S.c_max(e, l, assign, m) == opt
        assert opt >= S.lower_bound(e, l, m) - 1e-12
        assert S.c_max(e, l, S.lpt(e, l, m), m) >= opt
    for _ in range(40):                       # one stage only: Graham's bound holds
        n, m = rng.randint(1, 8), rng.randint(1, 3)
        e = [rng.randint(1, 9) for _ in range(n)]
        opt, _ = S.brute_force(e, [0] * n, m)
        assert S.c_max(e, [0] * n, S.lpt(e, [0] * n, m), m) <= (4 / 3 - 1 / (3 * m)) * opt + 1e-12


# ---------------------------------------------------------------------------------------------
# the library's scheduler against the oracle
# ---------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def B():
    import os
    from paper_2603_25120_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_25120_amd import build
        build.build()
    binding.lib()
    return binding


def test_library_lpt_matches_oracle_exactly(B):
    rng = np.random.default_rng(11)
    for n, m in ((0, 3), (1, 1), (7, 3), (64, 8), (500, 16), (2048, 64)):
        e = rng.lognormal(0.0, 1.0, n)
        l = rng.lognormal(0.5, 0.8, n)
        if n > 3:
            e[3] = e[1]; l[3] = l[1]           # exact ties
        got = B.mllm_schedule_lpt(e, l, m)
        assert list(got) == S.lpt(list(e), list(l), m)


def test_library_exact_matches_brute_force(B):
    rng = random.Random(3)
    for _ in range(60):
        n, m = rng.randint(1, 8), rng.randint(1, 3)
        e = [float(rng.randint(0, 12)) for _ in range(n)]
        l = [float(rng.randint(0, 12)) for _ in range(n)]
        assign, cmax, optimal = B.mllm_schedule(e, l, m, node_limit=10_000_000)
        opt, _ = S.brute_force(e, l, m)
        assert optimal
        assert cmax == opt == S.c_max(e, l, list(assign), m)


def test_library_hybrid_falls_back_to_lpt(B):
    rng = np.random.default_rng(2)
    e, l = rng.lognormal(0, 1, 400), rng.lognormal(0, 1, 400)
    assign, cmax, optimal = B.mllm_schedule(e, l, 16, node_limit=1000)
    lpt = S.lpt(list(e), list(l), 16)
    assert not optimal
    assert cmax <= S.c_max(list(e), list(l), lpt, 16) + 1e-12       # never worse than the fallback
    assert cmax == pytest.approx(S.c_max(list(e), list(l), list(assign), 16), rel=1e-12)
    assert min(assign) >= 0 and max(assign) < 16
    assert cmax >= S.lower_bound(list(e), list(l), 16) - 1e-12


def test_library_scheduler_argument_checks(B):
    with pytest.raises(B.MllmError) as err:
        B.mllm_schedule_lpt([1.0], [1.0], 0)
    assert err.value.status == 3
    with pytest.raises(B.MllmError) as err:
        B.mllm_schedule_lpt([1.0, -2.0], [1.0, 1.0], 2)
    assert err.value.status == 3
