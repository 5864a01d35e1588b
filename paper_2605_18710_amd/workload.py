"""Builds a stage of the synthetic workloads on the GPU: modules with seeded weights and
their staged input / upstream-gradient / target buffers (the decoupled form in which
modules are profiled and colocated: each module reads its own staged buffers, so the
modules of a stage are mutually independent, as the problem formulation requires).

Numbers only come from `synth`; all arithmetic runs in the library.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import binding as mb
from . import synth


def _fill_normal(module: mb.Module, name: str, seed: int, std: float) -> None:
    off, rows, cols = module.tensors[name]
    n = rows * cols
    # chunked so that the float64 temporaries stay small
    import torch
    from concurrent.futures import ThreadPoolExecutor
    step = 1 << 21
    # element i of the tensor is element i of the seed's stream; numpy releases the GIL
    # inside its loops, so chunks are drawn on a few host threads
    def draw(s):
        return s, synth.normal_range(seed, s, min(n, s + step), 0.0, std).astype(np.float32)
    with ThreadPoolExecutor(max_workers=8) as ex:
        for s, vals in ex.map(draw, range(0, n, step)):
            module.params[off + s:off + s + vals.size].copy_(torch.from_numpy(vals).to(module.tdtype))


def init_module_params(module: mb.Module, seed: int) -> None:
    """Matrices, tables and position rows N(0, 0.02); norm gains 1; biases 0."""
    module.params.zero_()
    for i, (name, (off, rows, cols)) in enumerate(module.tensors.items()):
        leaf = name.split(".")[-1]
        if leaf.startswith("w_") or leaf in ("table", "pos"):
            _fill_normal(module, name, seed + i, 0.02)
        elif leaf.endswith("_g"):
            module.params[off:off + rows * cols].fill_(1.0)


class StagedModule:
    """A module plus its staged device buffers."""

    def __init__(self, cfg: dict, dtype: str, seed: int, with_target: bool):
        import torch
        self.cfg = cfg
        self.module = mb.Module(cfg, dtype)
        init_module_params(self.module, seed)
        td = self.module.tdtype
        n_in, n_out = self.module.in_elems, self.module.out_elems
        mk = lambda sd, n, std: torch.from_numpy(synth.normal(sd, (n,), 0.0, std).astype(np.float32)).to(td).cuda()
        self.x = mk(seed + 900, n_in, 1.0)
        self.y = torch.empty(n_out, dtype=td, device="cuda")
        self.dx = torch.empty(n_in, dtype=td, device="cuda")
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        if with_target:
            self.target, self.dy = mk(seed + 901, n_out, 1.0), None
        else:
            # an upstream gradient of the size an MSE loss would produce
            self.target, self.dy = None, mk(seed + 902, n_out, 2.0 / n_out)

    def destroy(self):
        self.module.destroy()


class StagedStage:
    """All modules of one workload; `groups` lists which modules share a quota."""

    def __init__(self, config: int, dtype: str | None = None, layers_cap: int | None = None):
        wl = synth.WORKLOADS[config]
        self.wl = wl
        self.dtype = dtype or wl["dtype"]
        self.staged: List[StagedModule] = []
        self.names: List[str] = []
        for i, cfg in enumerate(wl["modules"]):
            cfg = dict(cfg)
            if layers_cap is not None and cfg["kind"] != "projector":
                cfg["layers"] = min(cfg["layers"], layers_cap)
            seed = synth.tensor_seed(config, 0) + 10000 * (i + 1)
            self.staged.append(StagedModule(cfg, self.dtype, seed, with_target=(cfg["kind"] == "decoder")))
            self.names.append(cfg["name"])
        self.groups = wl["groups"]
        self.batch = wl["modules"][0]["batch"]

    def group_of(self, name: str) -> int:
        for g, members in enumerate(self.groups):
            if name in members:
                return g
        raise KeyError(name)

    def plan_arrays(self, group_quotas):
        """Per-module quota/offset arrays from per-group quotas (groups packed from CU 0)."""
        offs, o = [], 0
        for q in group_quotas:
            offs.append(o)
            o += q
        quotas = [group_quotas[self.group_of(n)] for n in self.names]
        offsets = [offs[self.group_of(n)] for n in self.names]
        return quotas, offsets

    def reserve(self, group_quotas) -> None:
        o = 0
        for q in group_quotas:
            mb.pool_reserve(q, o, mb.STRIPED)
            o += q

    def run(self, group_quotas, mode=mb.COLOCATED) -> dict:
        if mode == mb.COLOCATED:
            quotas, offsets = self.plan_arrays(group_quotas)
        else:
            quotas, offsets = [group_quotas[0]] * len(self.names), [0] * len(self.names)
        s = self.staged
        return mb.stage_run([m.module for m in s], [m.x for m in s], [m.y for m in s], quotas, offsets,
                            mb.STRIPED, mode, dy=[m.dy for m in s], target=[m.target for m in s],
                            dx=[m.dx for m in s], loss=[m.loss for m in s])

    def flops(self) -> Dict[str, float]:
        return {m.cfg["name"]: synth.module_flops(m.cfg) for m in self.staged}

    def destroy(self):
        for m in self.staged:
            m.destroy()


class SplitStage:
    """The same workload with its decoder cut after layer k into two modules that read
    staged buffers like every other module.  An iteration is two stages (Eq. 1): stage A
    colocates the other groups with layers [0, k) under the given group quotas, stage B runs
    layers [k, L) alone on all CUs.  Cutting the decoder in time is a second way to balance an
    encoder against a decoder of several times its work (the slicing of modules the paper
    cites as prior work, Sec. 2.3, applied to one module and combined with its spatial
    sharing).  The streams of both stages are reserved once, here, as the engine of Sec. 3.2
    does before training; an iteration creates none and is timed by the host clock across
    both stages."""

    def __init__(self, config: int, k: int, group_quotas=None, dtype: str | None = None):
        wl = synth.WORKLOADS[config]
        self.dtype = dtype or wl["dtype"]
        self.groups = [list(g) for g in wl["groups"]]
        self.first: List[StagedModule] = []      # stage A, in workload order
        self.first_names: List[str] = []
        self.second: StagedModule | None = None  # stage B
        decoders = [m for m in wl["modules"] if m["kind"] == "decoder"]
        if len(decoders) != 1:
            raise ValueError("workload needs exactly one decoder to cut")
        if not 0 < k < decoders[0]["layers"]:
            raise ValueError("cut must leave layers on both sides")
        self.cus = mb.device_cu_count()
        self.group_quotas = list(group_quotas) if group_quotas is not None else list(wl["plans"][0])
        if len(self.group_quotas) != len(self.groups) or sum(self.group_quotas) > self.cus:
            raise ValueError("one quota per group, summing to at most the device's CUs")
        if len(set(self.group_quotas)) + 1 > mb.device_hw_queues():
            raise ValueError("the two stages need more streams than the process has hardware queues")
        for i, cfg in enumerate(wl["modules"]):
            seed = synth.tensor_seed(config, 0) + 10000 * (i + 1)
            if cfg["kind"] != "decoder":
                self.first.append(StagedModule(dict(cfg), self.dtype, seed, with_target=False))
                self.first_names.append(cfg["name"])
                continue
            a, b = dict(cfg), dict(cfg)
            a["layers"], b["layers"] = k, cfg["layers"] - k
            self.first.append(StagedModule(a, self.dtype, seed, with_target=True))
            self.first_names.append(cfg["name"])
            self.second = StagedModule(b, self.dtype, seed + 5000, with_target=True)
        # every stream both stages need, once (the streams of stage A plus the full-device one)
        self.offsets, o = [], 0
        for q in self.group_quotas:
            self.offsets.append(o)
            o += q
        mb.pool_clear()
        for q, off in zip(self.group_quotas, self.offsets):
            mb.pool_reserve(q, off, mb.STRIPED)
        mb.pool_reserve(self.cus, 0, mb.STRIPED)

    def _group_of(self, name: str) -> int:
        for g, members in enumerate(self.groups):
            if name in members:
                return g
        raise KeyError(name)

    def run(self) -> dict:
        import time
        import torch
        quotas = [self.group_quotas[self._group_of(n)] for n in self.first_names]
        offsets = [self.offsets[self._group_of(n)] for n in self.first_names]
        s, b = self.first, self.second
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ra = mb.stage_run([m.module for m in s], [m.x for m in s], [m.y for m in s], quotas, offsets, mb.STRIPED,
                          mb.COLOCATED, dy=[m.dy for m in s], target=[m.target for m in s],
                          dx=[m.dx for m in s], loss=[m.loss for m in s])
        rb = mb.stage_run([b.module], [b.x], [b.y], [self.cus], [0], mb.STRIPED, mb.TIME_SLICED,
                          dy=[b.dy], target=[b.target], dx=[b.dx], loss=[b.loss])
        wall = (time.perf_counter() - t0) * 1e3          # both calls block until their stage is done
        return dict(iteration_ms=wall, stage_ms=[ra["stage_ms"], rb["stage_ms"]],
                    module_ms=ra["module_ms"] + rb["module_ms"])

    def destroy(self):
        for m in self.first:
            m.destroy()
        self.second.destroy()
