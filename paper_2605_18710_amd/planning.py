"""Plans and runs a multi-module job on one GPU with the library's planner: measures each
module's time-vs-CU curve (the scaling surface of Sec. 3.3 restricted to one GPU), derives
the bandwidth-utilisation proxy, fits the interference coefficients of Eq. 8 from a few
colocated probe runs, forms stages with Alg. 1 and executes the stages one after another,
each colocated under its allocation.  The fit of Eq. 8, StageEval and Alg. 1 run in the
library; what is formed here, in Python, is bookkeeping around them: the utilisation
B(m, a) = work of a step / (measured time x peak) and the delay observations (differences
and ratios of measured times).  The work of a step is, by choice of `proxy`: "counters", the
HBM-side bytes that the L2's fabric counters read for one step of the module (a table under
profiles/, written from rocprofv3 runs; Sec. 3.3 profiles memory-bandwidth utilisation);
"bandwidth", the algorithmic bytes from `synth` where no counter reading exists; "compute",
the model FLOPs.
"""
from __future__ import annotations

import os
import statistics
from typing import Dict, List, Sequence, Tuple

from . import binding as mb
from . import synth
from .workload import StagedModule

PEAK_HBM_BYTES_PER_S = 8.0e12
PEAK_BF16_FLOPS = 2.5e15
STEP_BYTES_TABLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "module_step_hbm_bytes.txt")


def shape_signature(cfg: dict) -> str:
    """The key of a module in the table of measured step bytes."""
    if cfg["kind"] == "projector":
        return f"projector B{cfg['batch']} N{cfg['seq']} in{cfg['in_dim']} out{cfg['out_dim']}"
    return f"{cfg['kind']} B{cfg['batch']} N{cfg['seq']} h{cfg['hidden']} f{cfg['mlp']} L{cfg['layers']}"


def measured_step_bytes(path: str = STEP_BYTES_TABLE) -> Dict[str, float]:
    """shape signature -> HBM-side bytes (fetched + written) of one step, from the counter
    table; empty when the table is missing."""
    out: Dict[str, float] = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        cells = [c.strip() for c in line.split("|")]
        if len(cells) >= 6 and cells[0] == "bytes":
            out[cells[3]] = float(cells[4]) + float(cells[5])
    return out


class PlannedJob:
    """modules: list of module dicts (synth._enc / _dec / _proj form, unique names);
    edges: (producer name, consumer name) pairs.  Modules read staged buffers, so an edge
    only orders stages; it does not move data."""

    def __init__(self, modules: Sequence[dict], edges: Sequence[Tuple[str, str]], dtype: str = "bf16", seed: int = 18710000):
        self.cfgs = [dict(m) for m in modules]
        self.names = [m["name"] for m in self.cfgs]
        self.edges = [(self.names.index(a), self.names.index(b)) for a, b in edges]
        self.staged: List[StagedModule] = [
            StagedModule(cfg, dtype, seed + 10000 * (i + 1), with_target=(cfg["kind"] == "decoder"))
            for i, cfg in enumerate(self.cfgs)]
        self.cus = mb.device_cu_count()
        self.elem = 2 if dtype == "bf16" else 4
        self._probe_cache: Dict[tuple, dict] = {}     # colocated probe runs already measured

    # ------------------------------------------------------------------ measurement
    def _run(self, members: Sequence[int], quotas: Sequence[int], iters: int) -> dict:
        """Colocated run of `members` (module indices) at `quotas`, packed from CU 0; medians."""
        s = self.staged
        offsets, o = [], 0
        for q in quotas:
            offsets.append(o)
            o += q
        mb.pool_clear()            # a masked stream holds a hardware queue: keep only those in use
        for q, off in zip(quotas, offsets):
            mb.pool_reserve(q, off, mb.STRIPED)
        def once():
            return mb.stage_run([s[i].module for i in members], [s[i].x for i in members], [s[i].y for i in members],
                                list(quotas), offsets, mb.STRIPED, mb.COLOCATED,
                                dy=[s[i].dy for i in members], target=[s[i].target for i in members],
                                dx=[s[i].dx for i in members], loss=[s[i].loss for i in members])
        once()
        rs = [once() for _ in range(iters)]
        return dict(stage_ms=statistics.median(r["stage_ms"] for r in rs),
                    module_ms=[statistics.median(r["module_ms"][k] for r in rs) for k in range(len(members))])

    def measure_curves(self, grid: Sequence[int], iters: int = 3) -> List[List[float]]:
        """times[m][p]: module m alone on grid[p] CUs, ms."""
        return [[self._run([m], [q], iters)["stage_ms"] for q in grid] for m in range(len(self.staged))]

    def bandwidth_table(self, times: List[List[float]], proxy: str = "bandwidth") -> List[List[float]]:
        """B(m, a) in [0,1], the utilisation of Eq. 8.  "counters": the bytes the HBM-side
        counters read for one step of the module (measured once per shape on all CUs; the
        re-reads that make up most of them belong to the kernels, not to the quota), over the
        time the step took at quota a, against the HBM peak.  "bandwidth": the same with algorithmic
        bytes.  "compute": model FLOPs
        over the time, against the bf16 matrix peak -- on this GPU co-runners contend for the
        board's power budget before they contend for bandwidth, and matrix-core utilisation is
        the better stand-in for a module's share of that budget."""
        out = []
        table = measured_step_bytes() if proxy == "counters" else {}
        for cfg, row in zip(self.cfgs, times):
            if proxy == "counters":
                # a module whose shape was never profiled falls back to its algorithmic bytes
                w, peak = table.get(shape_signature(cfg), synth.module_bytes(cfg, self.elem)), PEAK_HBM_BYTES_PER_S
            elif proxy == "bandwidth":
                w, peak = synth.module_bytes(cfg, self.elem), PEAK_HBM_BYTES_PER_S
            elif proxy == "compute":
                w, peak = synth.module_flops(cfg), PEAK_BF16_FLOPS
            else:
                raise ValueError(f"unknown proxy {proxy!r}")
            out.append([min(1.0, w / (t * 1e-3) / peak) for t in row])
        return out

    def fit_interference(self, grid, times, bw, probes: Sequence[Dict[int, int]], iters: int = 3,
                         form: int = mb.DELAY_ABSOLUTE):
        """probes: list of {module index: CUs on the grid} with two or more modules each.  Every
        module of every probe gives one observation.  DELAY_ABSOLUTE (Eq. 7-8): the delay in ms
        (colocated time - time alone at the same quota) against the utilisations of all modules
        of the probe.  DELAY_PEER_RELATIVE: the delay as a fraction of the time alone, against
        the utilisations of the other modules of the probe.  Returns the fit of Eq. 8's
        expression, the additive-only fit and the observations."""
        groups, delays = [], []
        for pr in probes:
            members = sorted(pr)
            key = tuple(sorted(pr.items()))
            if key not in self._probe_cache:
                self._probe_cache[key] = self._run(members, [pr[m] for m in members], iters)
            r = self._probe_cache[key]
            bs = [bw[m][grid.index(pr[m])] for m in members]
            for k, m in enumerate(members):
                alone = times[m][grid.index(pr[m])]
                if form == mb.DELAY_ABSOLUTE:
                    groups.append(bs)
                    delays.append(r["module_ms"][k] - alone)
                else:
                    groups.append(bs[:k] + bs[k + 1:])
                    delays.append((r["module_ms"][k] - alone) / alone)
        e2, r2_2 = mb.interference_fit(groups, delays, mb.ADDITIVE)
        try:
            e3, r2_3 = mb.interference_fit(groups, delays, mb.COMPOSITE)
        except mb.MosaicError:       # e.g. only pairs probed in peer form: sum and product coincide
            e3, r2_3 = e2, r2_2
        return dict(e=e3, r2=r2_3, e_additive=e2, r2_additive=r2_2, n_obs=len(delays), groups=groups, delays=delays)

    # ---------------------------------------------------------------- plan and run
    def solve(self, grid, times, bw=None, e=None, flags=mb.EARLY_PRUNE | mb.CACHE, form=mb.DELAY_ABSOLUTE):
        return mb.planner_solve(len(self.staged), self.edges, list(grid), times, self.cus, bw=bw, e=e, flags=flags, form=form)

    def run_plan(self, stages: Sequence[Sequence[int]], alloc: Dict[int, int], iters: int = 3) -> dict:
        """Executes the stages one after another (Eq. 1); each stage colocated under its quotas."""
        per_stage = [self._run(list(st), [alloc[m] for m in st], iters)["stage_ms"] for st in stages]
        return dict(iteration_ms=sum(per_stage), stage_ms=per_stage)

    def destroy(self):
        mb.pool_clear()
        for s in self.staged:
            s.destroy()
