"""Oracle for the prefill batching plan and the iteration-time model -- TEST INFRASTRUCTURE ONLY.

LoongServe (arXiv 2404.09526), Sec. 5.3 "Batching" (the dynamic program over sorted requests and sorted
elastic instances) and Sec. 5.5 "Optimizations", analytical model based on SIB, Eq. 7 (iteration time = alpha + beta * sum(len)
+ gamma * sum(len^2), fitted by least squares).  Plain statements, written for checking by eye:

  * ``brute_force_plan`` enumerates EVERY way of cutting the request sequence and a prefix of the instance
    sequence into the same number of consecutive, non-empty pieces, keeps the cuts whose pieces respect the
    capacity constraint, prices each with ``plan_cost`` and returns the cheapest.  No recurrence, no pruning.
  * ``fit_model`` is the least-squares solution of the three-column linear system, by ``numpy.linalg.lstsq``.

Readings of the paper taken here (it leaves them open):
  * a batch's term T(R[j,i], E[l,k]) is the sum, over the requests of the batch, of the batch's iteration
    time divided by the request's input length (the "input latency" the section minimises is per input
    token, as in the gain / cost formulas of Sec. 5.1 and 5.2); the iteration time is the model of Sec. 5.5
    with the coefficients of the batch's degree of parallelism (its number of instances);
  * batches take consecutive requests and consecutive instances, both from the front; instances left over at
    the end stay unused (the minimum over the second index in the text);
  * D[j,i] <= V[l,k]: the tokens of the batch must fit the unused slots of its instances;
  * "trained by the least square method" (Sec. 5.5) says nothing about weighting: the fit takes optional
    per-sample weights; unweighted is the default.
Pinning status: pinned by tests/test_plan_oracle_pins.py (hand-priced cases, closed forms, monotonicity in
the resources, exact recovery of known coefficients).  The paper prints no numeric example for either.
"""
from __future__ import annotations

import itertools
from typing import List, Optional, Sequence, Tuple

import numpy as np


def iteration_time(lens: Sequence[int], coef: Sequence[float]) -> float:
    """Sec. 5.5, Eq. 7: alpha + beta * sum(len) + gamma * sum(len^2)."""
    a, b, g = coef
    return a + b * float(sum(lens)) + g * float(sum(int(x) * int(x) for x in lens))


def batch_cost(lens: Sequence[int], coef: Sequence[float]) -> float:
    """Sum over the batch's requests of iteration time / input length."""
    t = iteration_time(lens, coef)
    return sum(t / float(x) for x in lens)


def plan_cost(req_len: Sequence[int], free_slots: Sequence[int], coefs: Sequence[Sequence[float]],
              req_cuts: Sequence[int], inst_cuts: Sequence[int]) -> Optional[float]:
    """Cost of the plan whose batch b holds requests [req_cuts[b-1], req_cuts[b]) on instances
    [inst_cuts[b-1], inst_cuts[b]) (cuts start implicitly at 0); None if a batch does not fit its instances.
    coefs[d-1] = (alpha, beta, gamma) at degree of parallelism d."""
    total, r0, e0 = 0.0, 0, 0
    for r1, e1 in zip(req_cuts, inst_cuts):
        lens = req_len[r0:r1]
        if sum(lens) > sum(free_slots[e0:e1]):
            return None
        total += batch_cost(lens, coefs[e1 - e0 - 1])
        r0, e0 = r1, e1
    return total


def _compositions(n: int, parts: int):
    """All increasing cut tuples (c_1 < ... < c_parts = n) with c_1 >= 1."""
    for inner in itertools.combinations(range(1, n), parts - 1):
        yield inner + (n,)


def brute_force_plan(req_len: Sequence[int], free_slots: Sequence[int],
                     coefs: Sequence[Sequence[float]]) -> Tuple[Optional[float], List[int], List[int]]:
    """Cheapest plan by exhaustive enumeration: (cost, req_cuts, inst_cuts), cost None if nothing fits."""
    n, m = len(req_len), len(free_slots)
    best = (None, [], [])
    for k in range(1, m + 1):                      # instances used: the first k
        for parts in range(1, min(n, k) + 1):
            for rc in _compositions(n, parts):
                for ec in _compositions(k, parts):
                    c = plan_cost(req_len, free_slots, coefs, rc, ec)
                    if c is not None and (best[0] is None or c < best[0]):
                        best = (c, list(rc), list(ec))
    return best


def fit_model(sum_len: Sequence[float], sum_len_sq: Sequence[float], times: Sequence[float],
              weights: Optional[Sequence[float]] = None) -> np.ndarray:
    """Least-squares (alpha, beta, gamma) of time ~ alpha + beta * sum_len + gamma * sum_len_sq.  With weights,
    sample i's equation is multiplied by weights[i] first (weights = 1 / time minimises the relative residual)."""
    A = np.stack([np.ones(len(times)), np.asarray(sum_len, np.float64), np.asarray(sum_len_sq, np.float64)], axis=1)
    y = np.asarray(times, np.float64)
    if weights is not None:
        w = np.asarray(weights, np.float64)
        A, y = A * w[:, None], y * w
    sol, *_ = np.linalg.lstsq(A, y, rcond=None)
    return sol
