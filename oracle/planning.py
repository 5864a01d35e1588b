"""CPU checker ("oracle") for the planning side of temporal-spatial multiplexing on one GPU:
the I/O-interference correction of the performance model, the per-stage allocation
problem and the greedy stage-formation loop.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package.  It shares
no code with the C++ planner in the library.

What is written out here, and from where:

  * interference_delta / interference_fit -- Sec. 3.3, Eq. 7-8: the delay a module suffers
    on a GPU it shares is  e1 + e2 * sum_m B_m + e3 * prod_m B_m  over the bandwidth
    utilisations B_m in [0,1] of ALL modules placed on that GPU; the three coefficients are
    fitted to measured delays.  The paper does not name the fitting criterion; ordinary
    least squares is taken (it reports the coefficient of determination R^2, which is the
    least-squares figure of merit).  The "additive-only" comparison model drops the
    product term.  Fit = numpy.linalg.lstsq on the design matrix whose rows are
    [1, sum B, prod B].
  * stage_time / stage_eval -- Sec. 3.1, Eq. 4-5 (stage time = slowest module; quotas of
    the GPU sum to at most 1) with Eq. 7 (rectified time = grid-sampled time + delay).
    stage_eval is the definition: every assignment of one grid level per module is
    visited (itertools.product), the feasible one with the smallest stage time wins.
  * gahc -- Sec. 3.4, Alg. 1: every module starts as its own stage in a topological order;
    each round evaluates all pairs of stages whose merge keeps the stage order acyclic,
    takes the pair with the largest strictly positive saving T_x + T_y - T_xy, merges it,
    and stops when no pair saves time.  Early pruning and result caching (Sec. 3.4) change
    the amount of work, never the result, and are NOT part of this checker: the C++ planner
    has them and must agree with this plain loop with either switched on or off.

A second way of charging the delay is offered beside the paper's (it is this build's, not
the paper's): PEER_RELATIVE evaluates Eq. 8's expression over the utilisations of the OTHER
modules on the GPU and charges it as a fraction of the module's own time,
T_m * (1 + e1 + e2 * sum_{m' != m} B_m' + e3 * prod_{m' != m} B_m').  On the GPU this build
targets, co-runners slow a module down through the shared power budget, in proportion to
its own run time and to the co-runners' matrix-core utilisation, which the paper's one
additive term per GPU cannot express.

Readings where the paper is silent (the C++ planner takes the same ones):
  * a module alone on the GPU suffers no delay: Eq. 8 is applied only to stages of two or
    more modules (the grid-sampled time of a module already contains its own traffic);
  * ties: among assignments with equal stage time the lexicographically smallest tuple of
    grid-level indices (modules in ascending index order) wins; among pairs with equal
    saving the first in (x ascending, y ascending) order over the current stage list wins;
  * topological order: Kahn's algorithm, always taking the ready stage whose smallest
    module index is smallest; the stage list is put back into that order after a merge;
  * merging is legal when neither stage is reachable from the other in the stage graph
    (an edge runs from stage a to stage b when some module of a feeds some module of b):
    a direct edge would put dependent modules in one stage, a longer path would make the
    merged stage both precede and follow the stages on it;
  * a stage that does not fit (no assignment within the CU budget) has infinite time.

Pins (tests/test_oracle_planning.py): planted coefficients recovered exactly from
noise-free delays; the R^2 of a hand-computed three-point example; stage_eval against a
closed form for modules with T = w/a; gahc never worse than the all-singleton plan and
never better than a brute-force search over every legal ordered partition, equal to it
where greedy is provably optimal.  The paper prints no worked example for these steps.
"""
from __future__ import annotations

import itertools
import math
from typing import Dict, FrozenSet, List, Optional, Sequence, Tuple

import numpy as np

ADDITIVE, COMPOSITE = 0, 1
# how a fitted delay enters a module's time
ABSOLUTE, PEER_RELATIVE = 0, 1


# ------------------------------------------------------------------------ Eq. 7-8
def interference_delta(e: Sequence[float], bw: Sequence[float]) -> float:
    """Eq. 8 for one GPU: e1 + e2 * sum(B) + e3 * prod(B) over the modules on it."""
    s = 0.0
    p = 1.0
    for b in bw:
        s += b
        p *= b
    return e[0] + e[1] * s + e[2] * p


def interference_fit(groups: Sequence[Sequence[float]], delta: Sequence[float], model: int = COMPOSITE):
    """Least-squares coefficients (e1, e2, e3) of Eq. 8 and the fit's R^2.

    groups[i] lists the bandwidth utilisations of the modules that shared the GPU in
    observation i; delta[i] is the delay measured for one of them.  model = ADDITIVE drops
    the product term (e3 = 0)."""
    rows = []
    for g in groups:
        s = float(np.sum(np.asarray(g, dtype=np.float64)))
        p = float(np.prod(np.asarray(g, dtype=np.float64)))
        rows.append([1.0, s, p] if model == COMPOSITE else [1.0, s])
    X = np.asarray(rows, dtype=np.float64)
    y = np.asarray(delta, dtype=np.float64)
    coef, _, rank, _ = np.linalg.lstsq(X, y, rcond=None)
    if rank < X.shape[1]:
        raise ValueError("observations do not determine the coefficients")
    e = [float(coef[0]), float(coef[1]), float(coef[2]) if model == COMPOSITE else 0.0]
    pred = X @ coef
    ss_res = float(np.sum((y - pred) ** 2))
    ss_tot = float(np.sum((y - y.mean()) ** 2))
    r2 = 1.0 - ss_res / ss_tot if ss_tot > 0 else (1.0 if ss_res == 0 else -math.inf)
    return e, r2


# ------------------------------------------------------------------------ Eq. 4-5, 7
def stage_time(levels: Sequence[int], modules: Sequence[int], times, bw=None, e=None, form: int = ABSOLUTE) -> float:
    """Time of a stage whose module modules[k] runs at grid level levels[k]: the slowest
    module's rectified time.  ABSOLUTE (Eq. 7-8): grid-sampled time plus one delay computed
    over all modules of the stage.  PEER_RELATIVE: grid-sampled time times one plus the
    expression of Eq. 8 over the other modules of the stage.  A module alone is not delayed."""
    if e is None or bw is None or len(modules) < 2:
        return max(times[m][p] for m, p in zip(modules, levels))
    b = [bw[m][p] for m, p in zip(modules, levels)]
    if form == ABSOLUTE:
        d = interference_delta(e, b)
        return max(times[m][p] + d for m, p in zip(modules, levels))
    worst = -math.inf
    for k, (m, p) in enumerate(zip(modules, levels)):
        peers = b[:k] + b[k + 1:]
        worst = max(worst, times[m][p] * (1.0 + interference_delta(e, peers)))
    return worst


def stage_eval(modules: Sequence[int], cu_points: Sequence[int], times, cu_total: int, bw=None, e=None,
               form: int = ABSOLUTE):
    """Eq. 4-5 by definition: the assignment of one grid level per module, quotas summing
    to at most cu_total, that minimises the stage time.  Returns (time, {module: CUs});
    (inf, {}) when nothing fits."""
    modules = sorted(modules)
    best_t, best_levels = math.inf, None
    for levels in itertools.product(range(len(cu_points)), repeat=len(modules)):
        if sum(cu_points[p] for p in levels) > cu_total:
            continue
        t = stage_time(levels, modules, times, bw, e, form)
        if t < best_t:            # product() runs in lexicographic order: first minimum wins
            best_t, best_levels = t, levels
    if best_levels is None:
        return math.inf, {}
    return best_t, {m: cu_points[p] for m, p in zip(modules, best_levels)}


# --------------------------------------------------------------------------- Alg. 1
def _stage_edges(stages: List[FrozenSet[int]], edges) -> Dict[int, set]:
    where = {m: i for i, s in enumerate(stages) for m in s}
    out: Dict[int, set] = {i: set() for i in range(len(stages))}
    for a, b in edges:
        if where[a] != where[b]:
            out[where[a]].add(where[b])
    return out


def _reachable(adj: Dict[int, set], src: int, dst: int) -> bool:
    seen, stack = set(), [src]
    while stack:
        v = stack.pop()
        for w in adj[v]:
            if w == dst:
                return True
            if w not in seen:
                seen.add(w)
                stack.append(w)
    return False


def topo_order(stages: List[FrozenSet[int]], edges) -> List[FrozenSet[int]]:
    """Kahn's algorithm over the stage graph; among ready stages the one holding the
    smallest module index goes first."""
    adj = _stage_edges(stages, edges)
    indeg = {i: 0 for i in range(len(stages))}
    for a in adj:
        for b in adj[a]:
            indeg[b] += 1
    done: List[FrozenSet[int]] = []
    ready = [i for i in indeg if indeg[i] == 0]
    while ready:
        ready.sort(key=lambda i: min(stages[i]))
        i = ready.pop(0)
        done.append(stages[i])
        for b in adj[i]:
            indeg[b] -= 1
            if indeg[b] == 0:
                ready.append(b)
    if len(done) != len(stages):
        raise ValueError("dependency cycle")
    return done


def merge_is_legal(stages: List[FrozenSet[int]], edges, x: int, y: int) -> bool:
    adj = _stage_edges(stages, edges)
    return not _reachable(adj, x, y) and not _reachable(adj, y, x)


def gahc(n_modules: int, edges, cu_points, times, cu_total: int, bw=None, e=None, form: int = ABSOLUTE):
    """Alg. 1.  Returns (stages in execution order, {module: CUs}, iteration time)."""
    stages = topo_order([frozenset([m]) for m in range(n_modules)], edges)
    ev = {s: stage_eval(s, cu_points, times, cu_total, bw, e, form) for s in stages}
    while len(stages) > 1:
        best_gain, best = 0.0, None
        for x in range(len(stages)):
            for y in range(x + 1, len(stages)):
                if not merge_is_legal(stages, edges, x, y):
                    continue
                u = stages[x] | stages[y]
                if u not in ev:
                    ev[u] = stage_eval(u, cu_points, times, cu_total, bw, e, form)
                gain = ev[stages[x]][0] + ev[stages[y]][0] - ev[u][0]
                if gain > best_gain:
                    best_gain, best = gain, (x, y)
        if best is None:
            break
        x, y = best
        merged = stages[x] | stages[y]
        stages = topo_order([s for i, s in enumerate(stages) if i not in (x, y)] + [merged], edges)
    alloc: Dict[int, int] = {}
    t_iter = 0.0
    for s in stages:
        t_iter += ev[s][0]          # Eq. 1: stages follow one another in time
        alloc.update(ev[s][1])
    return stages, alloc, t_iter
