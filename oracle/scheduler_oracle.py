"""Plain CPU definition of the online microbatch scheduling problem and of the LPT heuristic.

TEST INFRASTRUCTURE ONLY (see stage_oracle.py): only tests and the benchmark's reporting may
import this file; the product never does and shares no code with it.

Problem (Online Microbatch Scheduler, "Problem Formulation"): a global batch of N items, item i
with an encoder-stage duration e[i] and an LLM-stage duration l[i]; assign every item to exactly
one of m buckets; bucket j's stage times are E_j = sum of e over its items and L_j = sum of l;
minimise C_max = max(max_j E_j, max_j L_j).

LPT ("Scheduling Optimization"): items in descending order of duration, each put into the bucket
with the lowest accumulated load.  The text leaves open what "duration" and "load" mean when an
item has two stage durations; the reading taken here: an item's duration is max(e[i], l[i]), a
bucket's load is max(E_j, L_j); ties go to the lower index (items and buckets).
"""
from __future__ import annotations

import itertools
from typing import List, Sequence, Tuple


def bucket_times(e: Sequence[float], l: Sequence[float], assign: Sequence[int], m: int) -> Tuple[List[float], List[float]]:
    E, L = [0.0] * m, [0.0] * m
    for i, j in enumerate(assign):       # items added in index order
        E[j] += e[i]
        L[j] += l[i]
    return E, L


def c_max(e, l, assign, m) -> float:
    """The objective: the largest stage time of any bucket."""
    E, L = bucket_times(e, l, assign, m)
    return max(max(E), max(L)) if m > 0 else 0.0


def lpt(e, l, m) -> List[int]:
    """Longest-processing-time-first assignment (bucket index per item)."""
    order = sorted(range(len(e)), key=lambda i: (-max(e[i], l[i]), i))
    E, L = [0.0] * m, [0.0] * m
    assign = [0] * len(e)
    for i in order:
        j = min(range(m), key=lambda b: (max(E[b], L[b]), b))
        assign[i] = j
        E[j] += e[i]
        L[j] += l[i]
    return assign


def brute_force(e, l, m) -> Tuple[float, List[int]]:
    """Exact optimum by enumerating all m^N assignments (tiny N only)."""
    best, best_assign = float("inf"), None
    for assign in itertools.product(range(m), repeat=len(e)):
        c = c_max(e, l, assign, m)
        if c < best:
            best, best_assign = c, list(assign)
    return best, best_assign


def lower_bound(e, l, m) -> float:
    """No assignment can beat the average load of either stage, nor the largest single item."""
    if not len(e):
        return 0.0
    return max(sum(e) / m, sum(l) / m, max(max(a, b) for a, b in zip(e, l)))
