"""CPU-only checks of the library's planning calls (interference fit, StageEval, the
stage-formation loop of Alg. 1) against the planning checker, on the same seeded inputs.
Integer results (stage composition, quotas) must be identical; times are sums and maxima
of the same doubles taken in the same order, so they are compared for equality too."""
import math

import numpy as np
import pytest

from oracle import planning as PL
from paper_2605_18710_amd import binding as mb
from paper_2605_18710_amd import synth


def random_job(seed, n, pts):
    u = synth.uniform(seed, (n, 6))
    times = [[0.2 + 4.0 * r[0] + (1.0 + 8.0 * r[1]) / min(a, pts[int(r[2] * len(pts)) % len(pts)]) for a in pts] for r in u]
    bw = [[min(1.0, 0.1 + 0.8 * r[3] * a / pts[-1]) for a in pts] for r in u]
    edges = [(a, b) for a in range(n) for b in range(a + 1, n) if u[a][4] * u[b][5] > 0.45]
    return times, bw, edges


def test_delta_matches_checker():
    for seed in range(5):
        b = list(synth.uniform(6000 + seed, (1 + seed,)))
        e = list(synth.normal(6100 + seed, (3,)))
        assert mb.interference_delta(e, b) == pytest.approx(PL.interference_delta(e, b), rel=1e-15, abs=1e-15)


@pytest.mark.parametrize("model", [PL.ADDITIVE, PL.COMPOSITE])
def test_fit_matches_checker(model):
    u = synth.uniform(6200, (50, 3))
    groups = [list(r[:2 + (i % 2)]) for i, r in enumerate(u)]
    noise = synth.normal(6201, (50,), 0.0, 0.05)
    delta = [0.2 + 1.1 * sum(g) + 3.0 * float(np.prod(g)) + z for g, z in zip(groups, noise)]
    e_ref, r2_ref = PL.interference_fit(groups, delta, model)
    e, r2 = mb.interference_fit(groups, delta, model)
    assert np.allclose(e, e_ref, rtol=1e-9, atol=1e-10)
    assert r2 == pytest.approx(r2_ref, abs=1e-10)
    assert 0.5 < r2 < 1.0


def test_fit_error_paths():
    with pytest.raises(mb.MosaicError):
        mb.interference_fit([[0.2, 0.3]] * 4, [1.0] * 4, mb.COMPOSITE)      # rank deficient
    with pytest.raises(mb.MosaicError):
        mb.interference_fit([[0.2], [0.3], []], [1.0, 2.0, 3.0], mb.ADDITIVE)  # empty group
    with pytest.raises(mb.MosaicError):
        mb.interference_fit([[0.2], [0.3]], [1.0, 2.0], 7)


@pytest.mark.parametrize("seed", range(10))
def test_stage_eval_matches_checker(seed):
    n = 2 + seed % 4
    pts = [32, 64, 96, 128, 160, 192, 224][: 4 + seed % 4]
    times, bw, _ = random_job(7000 + seed, n, pts)
    for members in ([0], list(range(n)), list(range(0, n, 2))):
        for kw in ({}, dict(bw=bw, e=[0.05, 0.3, 0.8]), dict(bw=bw, e=[0.02, 0.9, 0.4], form=PL.PEER_RELATIVE)):
            t_ref, a_ref = PL.stage_eval(members, pts, times, 256, **kw)
            t, a = mb.stage_eval(members, n, pts, times, 256, **kw)
            assert t == t_ref and a == a_ref, (members, kw.keys())


def test_stage_eval_infeasible_is_infinite():
    t, a = mb.stage_eval([0, 1, 2], 3, [128, 256], [[2.0, 1.0]] * 3, 256)
    assert math.isinf(t) and a == {}


@pytest.mark.parametrize("seed", range(16))
def test_planner_matches_checker_with_and_without_pruning_and_caching(seed):
    n = 2 + seed % 6
    pts = [32, 64, 128, 192, 224]
    times, bw, edges = random_job(8000 + seed, n, pts)
    for kw in ({}, dict(bw=bw, e=[0.05, 0.3, 0.8]), dict(bw=bw, e=[0.02, 0.9, 0.4], form=PL.PEER_RELATIVE)):
        st_ref, al_ref, t_ref = PL.gahc(n, edges, pts, times, 256, **kw)
        results = []
        for flags in (0, mb.EARLY_PRUNE, mb.CACHE, mb.EARLY_PRUNE | mb.CACHE):
            stages, alloc, t, stats = mb.planner_solve(n, edges, pts, times, 256, flags=flags, **kw)
            assert [sorted(s) for s in st_ref] == stages
            assert alloc == al_ref
            assert t == t_ref
            results.append(stats)
        # pruning and caching only ever remove work
        assert results[3]["stage_evals"] <= results[0]["stage_evals"]
        assert results[0]["cache_hits"] == 0 and results[0]["pruned"] == 0


def test_caching_and_pruning_save_work_on_a_wide_job():
    # seven independent modules that stop speeding up at 64 CUs: several rounds of merges,
    # each of which re-examines stage compositions seen in the round before
    n = 7
    pts = [32, 64, 128, 192, 224]
    w = synth.uniform(8100, (n,), 1.0, 3.0)
    times = [[float(w[m]) * 64.0 / min(a, 64) for a in pts] for m in range(n)]
    _, _, t0, s0 = mb.planner_solve(n, [], pts, times, 256, flags=0)
    _, _, t1, s1 = mb.planner_solve(n, [], pts, times, 256, flags=mb.EARLY_PRUNE | mb.CACHE)
    assert t0 == t1
    assert s1["cache_hits"] > 0 and s1["stage_evals"] < s0["stage_evals"]


def test_planner_error_paths():
    pts, times = [128, 256], [[2.0, 1.0]] * 2
    with pytest.raises(mb.MosaicError):
        mb.planner_solve(2, [(0, 1), (1, 0)], pts, times, 256)          # cycle
    with pytest.raises(mb.MosaicError):
        mb.planner_solve(2, [(0, 2)], pts, times, 256)                  # edge out of range
    with pytest.raises(mb.MosaicError):
        mb.planner_solve(17, [], pts, [[1.0, 1.0]] * 17, 256)           # too many modules
    with pytest.raises(mb.MosaicError):
        mb.planner_solve(2, [], pts, [[2.0, float("nan")], [1.0, 1.0]], 256)
