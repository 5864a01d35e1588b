"""Pins of the planning checker (oracle/planning.py) against things other than itself:
closed forms, hand-computed regressions, planted coefficients and a brute-force search
over every legal ordered partition.  The paper prints no worked example for these steps
(Sec. 3.3 Eq. 7-8, Sec. 3.1 Eq. 1-5, Sec. 3.4 Alg. 1)."""
import itertools
import math

import numpy as np
import pytest

from oracle import planning as PL
from paper_2605_18710_amd import synth


# ------------------------------------------------------------------------- Eq. 8
def test_delta_is_constant_plus_sum_plus_product():
    # 1 + 2*(0.5+0.2) + 3*(0.5*0.2) = 2.7 ; a transposed coefficient or a dropped term moves it
    assert PL.interference_delta([1.0, 2.0, 3.0], [0.5, 0.2]) == pytest.approx(2.7, abs=1e-15)
    # three modules: sum 1.0, product 0.024
    assert PL.interference_delta([0.5, 1.0, 10.0], [0.2, 0.3, 0.5]) == pytest.approx(0.5 + 1.0 + 0.3, abs=1e-15)
    # one module: sum = product = B
    assert PL.interference_delta([0.0, 1.0, 1.0], [0.25]) == pytest.approx(0.5, abs=1e-15)


def test_fit_recovers_planted_coefficients_exactly():
    u = synth.uniform(4101, (40, 3))
    groups = [list(r[:2]) if i % 3 else list(r) for i, r in enumerate(u)]
    e = [0.37, 1.9, -4.2]
    delta = [e[0] + e[1] * sum(g) + e[2] * float(np.prod(g)) for g in groups]
    got, r2 = PL.interference_fit(groups, delta, PL.COMPOSITE)
    assert np.allclose(got, e, rtol=0, atol=1e-10)
    assert r2 == pytest.approx(1.0, abs=1e-12)


def test_additive_fit_matches_simple_linear_regression_closed_form():
    # groups of two equal utilisations: x = sum B
    groups = [[0.1, 0.1], [0.2, 0.2], [0.4, 0.4], [0.45, 0.45]]
    x = np.array([0.2, 0.4, 0.8, 0.9])
    y = np.array([1.0, 2.0, 5.0, 7.0])
    slope = np.sum((x - x.mean()) * (y - y.mean())) / np.sum((x - x.mean()) ** 2)
    icpt = y.mean() - slope * x.mean()
    r = np.corrcoef(x, y)[0, 1]
    got, r2 = PL.interference_fit(groups, list(y), PL.ADDITIVE)
    assert got[0] == pytest.approx(icpt, abs=1e-12) and got[1] == pytest.approx(slope, abs=1e-12) and got[2] == 0.0
    assert r2 == pytest.approx(r * r, abs=1e-12)      # for a line with intercept R^2 is the squared correlation


def test_product_term_is_needed_when_delays_grow_with_the_product():
    u = synth.uniform(4102, (60, 2))
    groups = [list(r) for r in u]
    delta = [0.1 + 0.5 * sum(g) + 6.0 * g[0] * g[1] for g in groups]
    _, r2_add = PL.interference_fit(groups, delta, PL.ADDITIVE)
    _, r2_mul = PL.interference_fit(groups, delta, PL.COMPOSITE)
    assert r2_mul == pytest.approx(1.0, abs=1e-12)
    assert r2_add < 0.99


def test_fit_refuses_observations_that_do_not_span_the_model():
    with pytest.raises(ValueError):
        PL.interference_fit([[0.2, 0.3]] * 5, [1.0] * 5, PL.COMPOSITE)


# ----------------------------------------------------------------------- Eq. 4-5
def inverse_times(work, cu_points):
    """T_m(a) = w_m / a: the textbook perfectly-scaling module."""
    return [[w / a for a in cu_points] for w in work]


def test_stage_eval_hits_the_proportional_split():
    # continuous optimum of min max_m w_m/a_m s.t. sum a = A is a_m = A w_m / sum w, T = sum w / A
    pts = list(range(1, 9))
    t, alloc = PL.stage_eval([0, 1], pts, inverse_times([1.0, 3.0], pts), 8)
    assert t == pytest.approx(0.5, abs=1e-15) and alloc == {0: 2, 1: 6}
    t, alloc = PL.stage_eval([0, 1, 2], [1, 2, 3, 4, 5, 6], inverse_times([1.0, 2.0, 3.0], [1, 2, 3, 4, 5, 6]), 12)
    assert t == pytest.approx(0.5, abs=1e-15) and alloc == {0: 2, 1: 4, 2: 6}


def test_stage_eval_budget_and_infeasibility_and_ties():
    pts = [4, 8]
    times = [[2.0, 1.0], [2.0, 1.0], [2.0, 1.0]]
    assert PL.stage_eval([0, 1, 2], pts, times, 8) == (math.inf, {})          # 3 x 4 CUs > 8
    t, alloc = PL.stage_eval([0, 1], pts, times, 12)
    assert t == 2.0 and alloc == {0: 4, 1: 4}       # (4,8) and (8,4) tie at 2.0 with (4,4): smallest tuple wins
    t, alloc = PL.stage_eval([1], pts, times, 8)
    assert t == 1.0 and alloc == {1: 8}


def test_rectified_stage_time_adds_the_delay_to_shared_stages_only():
    pts = [2, 4, 6]
    times = inverse_times([2.0, 4.0], pts)
    bw = [[0.5, 0.5, 0.5], [0.2, 0.2, 0.2]]
    e = [0.25, 0.0, 0.0]
    t0, a0 = PL.stage_eval([0, 1], pts, times, 8)
    t1, a1 = PL.stage_eval([0, 1], pts, times, 8, bw, e)
    assert a0 == a1 and t1 == pytest.approx(t0 + 0.25, abs=1e-15)
    assert PL.stage_eval([0], pts, times, 8, bw, e)[0] == PL.stage_eval([0], pts, times, 8)[0]
    # a delay that grows with the co-runner's utilisation can move the optimum
    bw2 = [[0.1, 0.1, 0.1], [0.1, 0.5, 0.9]]
    t2, a2 = PL.stage_eval([0, 1], pts, times, 8, bw2, [0.0, 10.0, 0.0])
    assert t2 == pytest.approx(min(max(times[0][i], times[1][j]) + 10.0 * (bw2[0][i] + bw2[1][j])
                                   for i in range(3) for j in range(3) if pts[i] + pts[j] <= 8), abs=1e-15)


def test_peer_relative_delay_written_out():
    # two modules at fixed levels: module 0 is slowed by module 1's utilisation and vice versa
    times = [[10.0], [4.0]]
    bw = [[0.5], [0.2]]
    e = [0.1, 2.0, 0.0]
    t = PL.stage_time([0, 0], [0, 1], times, bw, e, PL.PEER_RELATIVE)
    assert t == pytest.approx(max(10.0 * (1 + 0.1 + 2.0 * 0.2), 4.0 * (1 + 0.1 + 2.0 * 0.5)), abs=1e-14)
    # three modules: module 2's peers are 0 and 1 (sum 0.7, product 0.1)
    times3, bw3 = [[1.0], [1.0], [5.0]], [[0.5], [0.2], [0.9]]
    t3 = PL.stage_time([0, 0, 0], [0, 1, 2], times3, bw3, [0.0, 1.0, 10.0], PL.PEER_RELATIVE)
    assert t3 == pytest.approx(5.0 * (1 + 0.7 + 10.0 * 0.1), abs=1e-14)
    # alone: no delay in either form
    assert PL.stage_time([0], [2], times3, bw3, [9.0, 9.0, 9.0], PL.PEER_RELATIVE) == 5.0


# ------------------------------------------------------------------------ Alg. 1
def set_partitions(items):
    if not items:
        yield []
        return
    first, rest = items[0], items[1:]
    for part in set_partitions(rest):
        for i in range(len(part)):
            yield part[:i] + [[first] + part[i]] + part[i + 1:]
        yield [[first]] + part


def brute_force_optimum(n, edges, pts, times, total, bw=None, e=None):
    """Eq. 1-3 by definition: the best sum of stage times over every partition of the
    modules into stages that can be ordered consistently with the dependencies."""
    best = math.inf
    for part in set_partitions(list(range(n))):
        stages = [frozenset(s) for s in part]
        try:
            PL.topo_order(stages, edges)
        except ValueError:
            continue
        where = {m: i for i, s in enumerate(stages) for m in s}
        if any(where[a] == where[b] for a, b in edges):
            continue
        # a stage may not hold two modules joined by a path either (checked on the closure)
        reach = {m: set() for m in range(n)}
        for _ in range(n):
            for a, b in edges:
                reach[a] |= {b} | reach[b]
        if any(where[a] == where[b] for a in range(n) for b in reach[a]):
            continue
        best = min(best, sum(PL.stage_eval(s, pts, times, total, bw, e)[0] for s in stages))
    return best


def check_plan(n, edges, stages, alloc, total):
    where = {m: i for i, s in enumerate(stages) for m in s}
    assert sorted(where) == list(range(n))                       # Eq. 2: every module placed once
    for a, b in edges:
        assert where[a] < where[b]                               # Eq. 3
    for s in stages:
        assert sum(alloc[m] for m in s) <= total                 # Eq. 5


def test_chain_cannot_merge_and_costs_the_sum_of_full_device_times():
    pts = [2, 4, 8]
    times = inverse_times([8.0, 16.0, 4.0], pts)
    stages, alloc, t = PL.gahc(3, [(0, 1), (1, 2)], pts, times, 8)
    assert [sorted(s) for s in stages] == [[0], [1], [2]]
    assert alloc == {0: 8, 1: 8, 2: 8} and t == pytest.approx(1.0 + 2.0 + 0.5, abs=1e-15)


def test_two_saturating_modules_merge_and_match_the_optimum():
    # neither module speeds up beyond 4 CUs, so sharing 8 CUs halves the iteration time
    pts = [2, 4, 8]
    times = [[4.0, 2.0, 2.0], [6.0, 3.0, 3.0]]
    stages, alloc, t = PL.gahc(2, [], pts, times, 8)
    assert [sorted(s) for s in stages] == [[0, 1]] and alloc == {0: 4, 1: 4} and t == 3.0
    assert brute_force_optimum(2, [], pts, times, 8) == 3.0


def test_perfectly_scaling_modules_gain_nothing_from_sharing():
    # T = w/a: the merged stage takes sum(w)/A, exactly the sum of the separate times: no strict saving
    pts = [2, 4, 6, 8]
    times = inverse_times([2.0, 6.0], pts)
    stages, _, t = PL.gahc(2, [], pts, times, 8)
    assert len(stages) == 2 and t == pytest.approx(1.0, abs=1e-15)


def test_merging_across_an_intermediate_stage_is_refused():
    # 0 -> 1 -> 2 and 3 free.  {0,2} would have to run both before and after 1.
    stages = [frozenset([0]), frozenset([1]), frozenset([2]), frozenset([3])]
    edges = [(0, 1), (1, 2)]
    assert not PL.merge_is_legal(stages, edges, 0, 2)
    assert not PL.merge_is_legal(stages, edges, 0, 1)
    assert PL.merge_is_legal(stages, edges, 0, 3) and PL.merge_is_legal(stages, edges, 2, 3)
    # path through a merged stage: {1,3} sits between 0 and 2 even though 3 touches neither
    stages = [frozenset([0]), frozenset([1, 3]), frozenset([2])]
    assert not PL.merge_is_legal(stages, edges, 0, 2)


@pytest.mark.parametrize("seed", range(12))
def test_random_jobs_are_valid_and_bracketed_by_singletons_and_brute_force(seed):
    n = 3 + seed % 3
    pts = [2, 4, 6, 8]
    u = synth.uniform(5200 + seed, (n, 6))
    # saturating curves: T = serial + w / min(a, knee)
    times = [[0.2 + 4.0 * r[0] + (1.0 + 8.0 * r[1]) / min(a, pts[int(r[2] * 4) % 4]) for a in pts] for r in u]
    bw = [[min(1.0, 0.1 + 0.8 * r[3] * a / 8.0) for a in pts] for r in u]
    edges = [(a, b) for a in range(n) for b in range(a + 1, n) if u[a][4] * u[b][5] > 0.45]
    for model in (None, [0.05, 0.3, 0.8]):
        kw = {} if model is None else dict(bw=bw, e=model)
        stages, alloc, t = PL.gahc(n, edges, pts, times, 8, **kw)
        check_plan(n, edges, stages, alloc, 8)
        singles = sum(min(times[m]) for m in range(n))
        best = brute_force_optimum(n, edges, pts, times, 8, **kw)
        assert best - 1e-12 <= t <= singles + 1e-12
        assert t == pytest.approx(sum(PL.stage_eval(s, pts, times, 8, **kw)[0] for s in stages), abs=1e-12)
