"""Pins of oracle/plan.py against things other than itself: hand-priced plans, closed forms, properties
that any correct planner has, and exact recovery of known model coefficients (Sec. 5.3 and 5.5)."""
import math

import numpy as np
import pytest

from oracle import plan


def test_iteration_time_is_the_three_term_model():
    # Sec. 5.5 (Eq. 7) with numbers worked by hand: 2 + 0.5 * (3 + 4) + 0.25 * (9 + 16) = 11.75
    assert plan.iteration_time([3, 4], (2.0, 0.5, 0.25)) == pytest.approx(11.75)
    assert plan.batch_cost([3, 4], (2.0, 0.5, 0.25)) == pytest.approx(11.75 / 3 + 11.75 / 4)


def test_two_requests_two_instances_priced_by_hand():
    # lengths 8 and 2; coefficients: one instance (0, 0, 1) -> time = sum of squares; two instances (0, 0, 0.5)
    # together on both instances: time 0.5 * 68 = 34 -> 34/8 + 34/2 = 21.25
    # together on the first instance alone: time 68 -> 8.5 + 34 = 42.5
    # separately, one instance each: 64/8 + 4/2 = 10          <- cheapest
    coefs = [(0.0, 0.0, 1.0), (0.0, 0.0, 0.5)]
    cost, rc, ec = plan.brute_force_plan([8, 2], [100, 100], coefs)
    assert cost == pytest.approx(10.0) and rc == [1, 2] and ec == [1, 2]
    assert plan.plan_cost([8, 2], [100, 100], coefs, [2], [2]) == pytest.approx(21.25)
    assert plan.plan_cost([8, 2], [100, 100], coefs, [2], [1]) == pytest.approx(42.5)


def test_capacity_forces_a_wider_batch():
    # the long request (8 tokens) does not fit one instance of 5 free slots: the only plan that fits puts both
    # requests on both instances (10 tokens <= 10 slots); price as above: 21.25
    coefs = [(0.0, 0.0, 1.0), (0.0, 0.0, 0.5)]
    cost, rc, ec = plan.brute_force_plan([8, 2], [5, 5], coefs)
    assert cost == pytest.approx(21.25) and rc == [2] and ec == [2]
    assert plan.brute_force_plan([8, 4], [5, 5], coefs)[0] is None          # 12 tokens never fit 10 slots


def test_constant_overhead_only_favours_one_request_per_instance():
    # time = 1 whatever the batch: cost = sum 1/len, the same for every plan that fits -> equals the closed form
    lens = [9, 7, 5, 3]
    coefs = [(1.0, 0.0, 0.0)] * 4
    cost, _, _ = plan.brute_force_plan(lens, [100] * 4, coefs)
    assert cost == pytest.approx(sum(1.0 / x for x in lens))


def test_linear_speedup_uses_every_instance_for_a_single_request():
    # one request, time = len^2 / d: the more instances the better; with m instances the cost is len / m
    coefs = [(0.0, 0.0, 1.0 / d) for d in range(1, 5)]
    cost, rc, ec = plan.brute_force_plan([12], [100] * 4, coefs)
    assert cost == pytest.approx(12.0 / 4) and rc == [1] and ec == [4]


def test_more_resources_never_cost_more():
    rng = np.random.default_rng(5)
    for _ in range(20):
        n, m = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        lens = sorted((int(x) for x in rng.integers(1, 50, n)), reverse=True)
        slots = [int(x) for x in rng.integers(20, 120, m + 1)]
        coefs = [(float(rng.uniform(0, 5)), float(rng.uniform(0, 1)), float(rng.uniform(0, 0.1)) / d) for d in range(1, m + 2)]
        a = plan.brute_force_plan(lens, slots[:m], coefs)[0]
        b = plan.brute_force_plan(lens, slots, coefs)[0]               # one more instance at the end
        if a is not None:
            assert b is not None and b <= a + 1e-12


def test_number_of_plans_enumerated_matches_the_count_of_compositions():
    # with everything fitting, plans of `parts` batches on the first k instances: C(n-1, parts-1) * C(k-1, parts-1)
    n, m = 4, 3
    count = sum(1 for k in range(1, m + 1) for parts in range(1, min(n, k) + 1)
                for _ in plan._compositions(n, parts) for _ in plan._compositions(k, parts))
    expect = sum(math.comb(n - 1, p - 1) * math.comb(k - 1, p - 1) for k in range(1, m + 1) for p in range(1, min(n, k) + 1))
    assert count == expect == 15


def test_fit_recovers_known_coefficients_and_a_textbook_line():
    rng = np.random.default_rng(11)
    lens = rng.integers(1000, 60000, size=12).astype(np.float64)
    t = 3e-5 + 2e-9 * lens + 7e-13 * lens * lens
    sol = plan.fit_model(lens, lens * lens, t)
    assert sol == pytest.approx([3e-5, 2e-9, 7e-13], rel=1e-6)
    # degenerate to ordinary linear regression when the quadratic column is zero: y = 1 + 2x through 3 exact points
    sol = plan.fit_model([0.0, 1.0, 2.0], [0.0, 0.0, 0.0], [1.0, 3.0, 5.0])
    assert sol[0] == pytest.approx(1.0) and sol[1] == pytest.approx(2.0)


def test_weighted_fit_reduces_to_textbook_cases():
    # weights (1, 1, 0): the third sample is ignored -> the line through the first two points exactly
    sol = plan.fit_model([0.0, 1.0, 5.0], [0.0, 0.0, 0.0], [1.0, 3.0, 100.0], weights=[1.0, 1.0, 0.0])
    assert sol[0] == pytest.approx(1.0) and sol[1] == pytest.approx(2.0)
    # equal weights change nothing
    rng = np.random.default_rng(2)
    x = rng.uniform(1, 9, 7); t = 1 + 2 * x + 0.5 * x * x + 0.01 * rng.standard_normal(7)
    assert plan.fit_model(x, x * x, t, weights=[3.0] * 7) == pytest.approx(plan.fit_model(x, x * x, t), rel=1e-9)
    # constant model, weights 1/t: minimising sum((a - t_i)^2 / t_i^2) gives a = sum(1/t) / sum(1/t^2)
    t = np.array([1.0, 2.0, 4.0])
    sol = plan.fit_model([0.0] * 3, [0.0] * 3, t, weights=1 / t)
    assert sol[0] == pytest.approx((1 / t).sum() / (1 / t ** 2).sum())
