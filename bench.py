#!/usr/bin/env python3
"""Benchmark of the multiplexed stage on one MI355X.

A step is one forward+backward of every module of the workload (all hot-path kernels) over
one batch of synthetic input, run under the best measured plan: stages one after another,
the modules of a stage side by side on disjoint CU quotas.  The same modules are also run
time-sliced (every module alone on all CUs, one after another); the line printed at the
end carries both, every plan that was measured, the per-module MFMA utilisation at quota,
the roofline of the dominant kernel and the CPU checker's time on a bounded sample.  The
default workload is the largest one that fits one GPU (vision + audio + 7B-shaped decoder);
the CLIP-B / small-LM workload is reported beside it under "secondary".

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--secondary 1]
    python bench.py --roofline-only | --attention-only | --bandwidth-only
                                         # only that kernel loop (the commands profiled in profiles/)
    python bench.py --power-only | --library-only
                                         # context: board power and clock under the GEMM; the GEMM beside the vendor library
    python bench.py --layer-split        # also the two-stage plan with the decoder cut in time
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def time_kernel(fn, reps, warm=3, settle_ms=0.0):
    """Average duration in ms of `reps` launches of fn on the default stream (HIP events
    recorded on that same stream).  settle_ms > 0: after the warm-up calls, fn is launched
    untimed for about that long first.  From idle the board runs the first ~1.5 ms of heavy
    work above its sustained clock, then the power controller clamps below it and settles
    over the next ~15 ms; a training step sees the settled rate, so that is what is timed."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    if settle_ms > 0.0:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            fn()
        e1.record()
        torch.cuda.synchronize()
        est = max(e0.elapsed_time(e1) / 3.0, 1e-3)
        for _ in range(int(settle_ms / est) + 1):
            fn()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


PROFILE_OF_SHAPE = {(8192, 2048, 11264): "gemm_bf16_kernel_roofline_config2.txt",
                    (32768, 4096, 22016): "gemm_bf16_kernel_roofline_7b_shape.txt"}


def profiled_traffic(form, shape):
    """HBM bytes per launch of the roofline kernel, from the committed rocprofv3 --pmc summary of
    that shape (FETCH_SIZE / WRITE_SIZE scaled by a copy of known size); None if there is none."""
    name = PROFILE_OF_SHAPE.get(tuple(shape))
    if name is None:
        return None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch:"):
                vals = dict(kv.split("=") for kv in line.split(":", 1)[1].split())
                return int(vals[form])
    except (OSError, KeyError, ValueError):
        pass
    return None


def roofline_gemm(mb, T, k, n, reps, settle_ms):
    """The dominant kernel: the bf16 MFMA GEMM at the decoder's gate/up projection shape,
    forward, input-gradient and weight-gradient forms, on all CUs, each timed after
    settle_ms of untimed calls (see time_kernel)."""
    import torch
    bf = torch.bfloat16
    X = torch.randn(T, k, device="cuda", dtype=bf)
    W = (torch.randn(k, n, device="cuda", dtype=torch.float32) * 0.02).to(bf)
    dY = torch.randn(T, n, device="cuda", dtype=bf)
    Y = torch.empty(T, n, device="cuda", dtype=bf)
    dX = torch.empty(T, k, device="cuda", dtype=bf)
    dW = torch.empty(k, n, device="cuda", dtype=bf)
    ws = torch.empty(mb.linear_wgrad_scratch_bytes(T, k, n), dtype=torch.uint8, device="cuda")
    q = mb.device_cu_count()
    flops = 2.0 * T * k * n
    out = {}
    out["fprop"] = time_kernel(lambda: mb.op_linear_fwd(None, q, "bf16", T, k, n, X, W, None, None, Y), reps, 3, settle_ms)
    out["dgrad"] = time_kernel(lambda: mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY, W, None, dX), reps, 3, settle_ms)
    out["wgrad"] = time_kernel(lambda: mb.op_linear_wgrad(None, q, "bf16", T, k, n, X, dY, dW, None, ws), reps, 3, settle_ms)
    return flops, out


def bandwidth_kernels(mb, T, h, f, reps):
    """Achieved HBM GB/s of the bandwidth-bound kernels at the decoder's shapes
    (algorithmic bytes: norm fwd 4 B/elem, norm bwd with residual 8 B/elem, SwiGLU fwd
    6 B per output elem, SwiGLU bwd 10 B)."""
    import torch
    bf = torch.bfloat16
    q = mb.device_cu_count()
    x = torch.randn(T, h, device="cuda", dtype=bf); g = torch.ones(h, device="cuda", dtype=bf)
    y = torch.empty_like(x); st = torch.empty(T, 2, device="cuda", dtype=torch.float32)
    dy = torch.randn(T, h, device="cuda", dtype=bf); dx = torch.empty_like(x); dg = torch.empty_like(g)
    sc = torch.empty(mb.norm_bwd_scratch_bytes(h), dtype=torch.uint8, device="cuda")
    gu = torch.randn(T, 2 * f, device="cuda", dtype=bf); a = torch.empty(T, f, device="cuda", dtype=bf)
    da = torch.randn(T, f, device="cuda", dtype=bf); dgu = torch.empty_like(gu)
    res = {}
    ms = time_kernel(lambda: mb.op_norm_fwd(None, q, "bf16", "rmsnorm", T, h, 1e-5, x, g, None, y, st), reps)
    res["rmsnorm_fwd"] = 4.0 * T * h / ms / 1e6
    ms = time_kernel(lambda: mb.op_norm_bwd(None, q, "bf16", "rmsnorm", T, h, x, g, st, dy, dy, dx, dg, None, sc), reps)
    res["rmsnorm_bwd"] = 8.0 * T * h / ms / 1e6
    ms = time_kernel(lambda: mb.op_swiglu_fwd(None, q, "bf16", T, f, gu, a), reps)
    res["swiglu_fwd"] = 6.0 * T * f / ms / 1e6
    ms = time_kernel(lambda: mb.op_swiglu_bwd(None, q, "bf16", T, f, gu, da, dgu), reps)
    res["swiglu_bwd"] = 10.0 * T * f / ms / 1e6
    # layer variants: rotary embedding in place on q|k of [T, 3h] (4 B per q|k element), AdamW
    # on bf16 parameters with fp32 moments (read p, g, m, v; write p, m, v: 22 B per element)
    H = max(1, h // 128)
    qkv = torch.randn(T, 3 * h, device="cuda", dtype=bf)
    table = torch.empty(mb.rope_table_bytes(T, 128), dtype=torch.uint8, device="cuda")
    mb.op_rope_table(None, q, T, 128, 10000.0, table)
    ms = time_kernel(lambda: mb.op_rope(None, q, "bf16", 1, T, H, 128, 1, qkv, table), reps)
    res["rope"] = 4.0 * T * 2 * H * 128 / ms / 1e6
    n = h * 2 * f
    p_ = torch.randn(n, device="cuda", dtype=bf); g_ = torch.randn(n, device="cuda", dtype=bf)
    m_ = torch.zeros(n, device="cuda", dtype=torch.float32); v_ = torch.zeros_like(m_)
    ms = time_kernel(lambda: mb.op_adamw(None, q, "bf16", n, p_, g_, m_, v_, None, 1e-4, 0.9, 0.999, 1e-8, 0.01, 7), reps)
    res["adamw"] = 22.0 * n / ms / 1e6
    return {k: round(v, 1) for k, v in res.items()}


def attention_kernels(mb, B, N, H, d, causal, reps):
    """Flash-style attention forward and backward at the decoder's shape; TFLOP/s with model
    FLOPs (4*B*N^2*h forward, halved under the causal mask; backward = 2x forward)."""
    import torch
    bf = torch.bfloat16
    q = mb.device_cu_count()
    h = H * d
    qkv = torch.randn(B * N, 3 * h, device="cuda", dtype=bf)
    O = torch.empty(B * N, h, device="cuda", dtype=bf); dO = torch.randn(B * N, h, device="cuda", dtype=bf)
    lse = torch.empty(B * H * N, device="cuda", dtype=torch.float32); delta = torch.empty_like(lse)
    dqkv = torch.empty_like(qkv)
    tf = time_kernel(lambda: mb.op_attention_fwd(None, q, "bf16", B, N, H, d, causal, qkv, O, lse), reps, 3, 40.0)
    tb = time_kernel(lambda: mb.op_attention_bwd(None, q, "bf16", B, N, H, d, causal, qkv, O, lse, dO, dqkv, delta), reps, 3, 40.0)
    fl = 4.0 * B * N * N * h * (0.5 if causal else 1.0)
    return dict(shape=dict(B=B, N=N, H=H, d=d, causal=causal), fwd_ms=round(tf, 4), bwd_ms=round(tb, 4),
                fwd_tflops=round(fl / tf / 1e9, 1), bwd_tflops=round(2.0 * fl / tb / 1e9, 1))


def power_probe(mb, seconds=3.0):
    """Board power and shader clock while a GEMM of the 7B-shaped gate/up projection
    (T=32768, k=4096, n=22016) runs in a loop: this build's forward form on N(0,1) inputs and
    on constant inputs (no bit toggling in the operands), its two gradient forms, and, as
    context, torch.matmul (the vendor library) with the weight stored k x n ("nn") and
    n x k ("nt").  Power and clock are read from the driver's sysfs files every 0.1 s by a
    host thread; missing files give nulls."""
    import glob
    import threading
    import torch
    bf = torch.bfloat16
    q = mb.device_cu_count()
    T, k, n = 32768, 4096, 22016
    X = torch.randn(T, k, device="cuda", dtype=bf)
    W = (torch.randn(k, n, device="cuda", dtype=torch.float32) * 0.02).to(bf)
    Wt = W.t().contiguous()
    dY = torch.randn(T, n, device="cuda", dtype=bf)
    Y = torch.empty(T, n, device="cuda", dtype=bf)
    dX = torch.empty(T, k, device="cuda", dtype=bf)
    dW = torch.empty(k, n, device="cuda", dtype=bf)
    ws = torch.empty(max(mb.linear_wgrad_scratch_bytes(T, k, n), 16), dtype=torch.uint8, device="cuda")
    pw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
    cap = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap"))
    clk = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))

    def read_w(paths):
        try:
            return int(open(paths[0]).read()) / 1e6
        except (OSError, ValueError, IndexError):
            return None

    def read_mhz():
        try:
            for line in open(clk[0]).read().splitlines():
                if line.strip().endswith("*"):
                    return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            pass
        return None

    fwd = lambda: mb.op_linear_fwd(None, q, "bf16", T, k, n, X, W, None, None, Y)
    cases = (("normal", fwd), ("dgrad", lambda: mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY, W, None, dX)),
             ("wgrad", lambda: mb.op_linear_wgrad(None, q, "bf16", T, k, n, X, dY, dW, None, ws)),
             ("library_nn", lambda: torch.matmul(X, W, out=Y)), ("library_nt", lambda: torch.matmul(X, Wt.t(), out=Y)),
             ("constant", fwd))
    out = {"shape": [T, k, n], "power_cap_w": read_w(cap)}
    for label, fn in cases:
        if label == "constant":
            X.fill_(1.0); W.fill_(0.5)
        watts, mhz, stop = [], [], []

        def poll():
            while not stop:
                watts.append(read_w(pw)); mhz.append(read_mhz())
                time.sleep(0.1)
        th = threading.Thread(target=poll)
        th.start()
        rates = []
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            rates.append(2.0 * T * k * n / time_kernel(fn, 20, 0) / 1e9)
        stop.append(1)
        th.join()
        half = len(watts) // 2           # the second half of the loop: the controller has settled
        ws_ = [w for w in watts[half:] if w is not None]
        ms = [m for m in mhz[half:] if m is not None]
        out[label] = {"tflops": round(statistics.median(rates[len(rates) // 2:]), 1),
                      "power_w": round(statistics.median(ws_), 1) if ws_ else None,
                      "sclk_mhz": round(statistics.median(ms), 1) if ms else None}
    return out


def library_compare(mb, reps=50, settle_ms=40.0):
    """Context only: the forward GEMM of this build beside torch.matmul (the vendor library)
    on the same N(0,1) inputs, timed the same way, in TFLOP/s.  "nn": weight stored k x n
    (this build's layout); "nt": weight stored n x k (a layout the boundary does not use)."""
    import torch
    bf = torch.bfloat16
    q = mb.device_cu_count()
    rows = []
    for (T, k, n) in ((8192, 2048, 11264), (8192, 2048, 2048), (8192, 5632, 2048), (32768, 4096, 22016),
                      (4608, 1024, 4096), (4608, 1024, 1024)):
        X = torch.randn(T, k, device="cuda", dtype=bf)
        W = (torch.randn(k, n, device="cuda", dtype=torch.float32) * 0.02).to(bf)
        Wt = W.t().contiguous()
        Y = torch.empty(T, n, device="cuda", dtype=bf)
        Y2 = torch.empty(T, n, device="cuda", dtype=bf)
        fl = 2.0 * T * k * n
        row = {"T": T, "k": k, "n": n}
        for name, fn in (("mosaic_fprop", lambda: mb.op_linear_fwd(None, q, "bf16", T, k, n, X, W, None, None, Y)),
                         ("library_nn", lambda: torch.matmul(X, W, out=Y2)),
                         ("library_nt", lambda: torch.matmul(X, Wt.t(), out=Y2))):
            row[name] = round(fl / time_kernel(fn, reps, 3, settle_ms) / 1e9, 1)
        row["max_abs_diff"] = float((Y.float() - Y2.float()).abs().max())
        rows.append(row)
        del X, W, Wt, Y, Y2
    return rows


def stream_pool_latency(mb, cus, repeats=30):
    """Analogue of the paper's stream-pool experiment (Sec. 5.3.1): latency of creating and
    destroying a quota'd stream on demand, for quotas 0.1 .. 0.9 of the device, against
    taking the same stream from the pre-created pool."""
    create, pooled = [], []
    for tenth in range(1, 10):
        q = max(8, round(cus * tenth / 10))
        for _ in range(repeats):
            t0 = time.perf_counter()
            s = mb.Stream(q, 0, mb.STRIPED)
            s.destroy()
            create.append((time.perf_counter() - t0) * 1e3)
        mb.pool_reserve(q, 0, mb.STRIPED)
        for _ in range(repeats):
            t0 = time.perf_counter()
            mb.pool_get(q, 0, mb.STRIPED)
            pooled.append((time.perf_counter() - t0) * 1e3)
    return dict(on_demand_create_destroy_ms=round(statistics.mean(create), 4),
                on_demand_max_ms=round(max(create), 4), pooled_get_ms=round(statistics.mean(pooled), 5),
                quotas="0.1..0.9 of the CUs, %d repeats each" % repeats)


def cpu_baseline(wl, budget_tflop=6.0):
    """The CPU checker as it stands, timed on this host on a bounded sample of the same
    workload: one layer of every encoder and decoder, forward+backward in float64, at full
    sequence length and hidden sizes, on as many samples of the batch as fit in about
    `budget_tflop` of arithmetic per module (all of them for the small modules, one or two for a
    7B-shaped decoder layer); the stage time is extrapolated as sample time x (batch / sampled
    batch) x layers.  Reported, not a target."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle import layers as O
    from paper_2605_18710_amd import synth
    from helpers import layer_params
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    total = 0.0
    parts = []
    for m in wl["modules"]:
        if m["kind"] == "projector":
            continue
        cfg = dict(m)
        per_sample = synth.module_flops(dict(cfg, batch=1, layers=1))
        b = int(max(1, min(cfg["batch"], budget_tflop * 1e12 // per_sample)))
        cfg["batch"] = b
        T, h = b * cfg["seq"], cfg["hidden"]
        x = synth.normal(124, (T, h)); dy = synth.normal(125, (T, h))
        p = layer_params(cfg, 123, perturb=False)
        t0 = time.perf_counter()
        y, saved = O.layer_fwd(x, p, cfg)
        O.layer_bwd(dy, p, saved, cfg)
        spent = time.perf_counter() - t0
        total += spent * (m["batch"] / b) * m["layers"]
        parts.append(f"{m['name']}: 1 of {m['layers']} layers at batch {b} of {m['batch']} in {spent:.2f}s")
    B = wl["modules"][0]["batch"]
    return dict(value=round(B / total, 5), unit="samples/s", cores=int(cores), kind="oracle",
                sample="float64 numpy forward+backward; " + "; ".join(parts) +
                       "; stage time extrapolated as sum(sample time x batch/sampled batch x layers), projector omitted")


def candidate_quotas(t_full_ms, t_budget_ms, cus, lo=8, max_points=11):
    """Quotas at which a module is worth measuring alone.  From the smallest at which it could
    still finish within t_budget_ms if its time scaled as 1/CUs: steps of 8 CUs below 64 (a
    quota below 32 CUs, or a multiple of 32, has all its CUs busy at once; any other keeps only
    the multiple of 32 below it busy, so the fine steps matter for the small modules only), then
    multiples of 32, plus 240 and 248 to show what the large module gets from the last CUs."""
    q_min = max(lo, int(t_full_ms * cus / t_budget_ms) // 8 * 8)
    top = [cus - 16, cus - 8] if q_min >= cus // 2 else []
    qs = [q for q in list(range(8, 64, 8)) + list(range(64, cus, 32)) + top if q_min <= q < cus]
    qs = sorted(set(qs))
    while len(qs) > max_points:          # drop the densest interior point
        gaps = [(qs[i + 1] - qs[i - 1], i) for i in range(1, len(qs) - 1) if qs[i] % 32]
        if not gaps:
            break
        qs.pop(min(gaps)[1])
    return qs


def module_steps(mb, synth, config, name, steps, warmup):
    """`warmup + steps` forward+backward steps of one module of the workload alone on all CUs
    and nothing else: under `rocprofv3 --kernel-trace --stats` the per-kernel totals divided by
    the number of steps are the kernel mix of one step."""
    from paper_2605_18710_amd.workload import StagedStage
    stage = StagedStage(config)
    if name not in stage.names:
        raise SystemExit(f"workload {config} has modules {stage.names}, not {name!r}")
    i = stage.names.index(name)
    m = stage.staged[i]
    cus = mb.device_cu_count()
    mb.pool_reserve(cus, 0, mb.STRIPED)
    ms = []
    for k in range(warmup + steps):
        r = mb.stage_run([m.module], [m.x], [m.y], [cus], [0], mb.STRIPED, mb.TIME_SLICED, dy=[m.dy], target=[m.target], dx=[m.dx], loss=[m.loss])
        if k >= warmup:
            ms.append(r["module_ms"][0])
    stage.destroy()
    mb.pool_clear()
    return {"workload": synth.WORKLOADS[config]["name"], "module": name, "steps_run": warmup + steps, "timed": steps,
            "ms_per_step": round(statistics.median(ms), 4), "min_ms": round(min(ms), 4)}


def measure_workload(mb, synth, config, steps, warmup, forced=None, layer_split=False):
    """Builds the staged workload `config`, measures the time-sliced baseline, the time-vs-CU
    curves, every named plan plus the plans derived from the curves (three-way, two modules
    sharing a quota, and the planner's stages), then times `steps` iterations of the best one."""
    import torch
    from paper_2605_18710_amd.workload import StagedStage
    wl = synth.WORKLOADS[config]
    cus = mb.device_cu_count()
    stage = StagedStage(config)
    B = stage.batch
    flops = stage.flops()
    names = stage.names
    ngroups = len(stage.groups)
    gflop = [sum(flops[n] for n in g) for g in stage.groups]
    gidx = [[i for i, n in enumerate(names) if n in g] for g in stage.groups]
    s = stage.staged
    med = statistics.median

    def run_groups(groups, quotas, offsets, mode):
        """One stage: the modules of `groups` (group indices), group g on (quotas[g], offsets[g])."""
        idx = [i for g in groups for i in gidx[g]]
        qs = [quotas[groups.index(stage.group_of(names[i]))] for i in idx]
        os_ = [offsets[groups.index(stage.group_of(names[i]))] for i in idx]
        r = mb.stage_run([s[i].module for i in idx], [s[i].x for i in idx], [s[i].y for i in idx], qs, os_, mb.STRIPED, mode,
                         dy=[s[i].dy for i in idx], target=[s[i].target for i in idx],
                         dx=[s[i].dx for i in idx], loss=[s[i].loss for i in idx])
        per_group = [sum(r["module_ms"][k] for k, i in enumerate(idx) if i in gidx[g]) for g in groups]
        return r["stage_ms"], per_group

    def reserve(plan):
        """Only the streams of the plan under test are alive: every masked stream owns a hardware
        queue, the process has few of them, and streams that share one run one after the other."""
        mb.pool_clear()
        for st in plan["stages"]:
            for q, o in set(zip(st["quotas"], st["offsets"])):
                mb.pool_reserve(q, o, mb.STRIPED)

    def run_plan(plan):
        """One iteration: the plan's stages one after another (Eq. 1), each colocated (Eq. 4)."""
        tot, per_group = 0.0, [0.0] * ngroups
        for st in plan["stages"]:
            mode = mb.COLOCATED if len(st["groups"]) > 1 else mb.TIME_SLICED
            ms, pg = run_groups(st["groups"], st["quotas"], st["offsets"], mode)
            tot += ms
            for g, v in zip(st["groups"], pg):
                per_group[g] = v
        return tot, per_group

    def median_plan(plan, iters):
        reserve(plan)
        run_plan(plan)
        rs = [run_plan(plan) for _ in range(iters)]
        return med(r[0] for r in rs), [med(r[1][g] for r in rs) for g in range(ngroups)]

    def pack(quotas):
        """Offsets for quotas that share the device: the largest quota starts at CU 0 (a CU range
        that starts at a multiple of 32 spreads over an XCD's shader engines in the order the
        dispatcher fills them, so all of its CUs are used at once; the small quotas at the top
        of the device are short enough not to care)."""
        offs, o = [0] * len(quotas), 0
        for i in sorted(range(len(quotas)), key=lambda i: -quotas[i]):
            offs[i] = o
            o += quotas[i]
        return offs

    def packed(quotas, label):
        return dict(label=label, stages=[dict(groups=list(range(ngroups)), quotas=list(quotas), offsets=pack(quotas))])

    # time-sliced baseline: every module alone on all CUs, back to back (sum over stages, Eq. 1)
    ts_plan = dict(label="time-sliced", stages=[dict(groups=[g], quotas=[cus], offsets=[0]) for g in range(ngroups)])
    ts_ms, group_ms_full = median_plan(ts_plan, 5)

    # time-vs-CU curves on multiples of 8 CUs, each module where it could still be useful
    grid = list(range(8, cus, 8))
    curves = [[1e30] * len(grid) for _ in range(ngroups)]
    for g in range(ngroups):
        for q in candidate_quotas(group_ms_full[g], 1.25 * ts_ms, cus):
            one = dict(label="curve", stages=[dict(groups=[g], quotas=[q], offsets=[0])])
            curves[g][grid.index(q)] = median_plan(one, 2)[0]
    chosen, predicted = mb.plan_choose(grid, curves, cus)

    # the paper's granularity (Sec. 3.4: quotas in steps of 10 % of the device): curves on the
    # multiples of 8 CUs nearest to the deciles, and the split chosen from those alone
    deciles = sorted({int(round(cus * d / 10.0 / 8.0)) * 8 for d in range(1, 10)})
    dcurves = [[1e30] * len(deciles) for _ in range(ngroups)]
    for g in range(ngroups):
        q_min = group_ms_full[g] * cus / (1.25 * ts_ms)
        for i, q in enumerate(deciles):
            if q < q_min:
                continue
            if q in grid and curves[g][grid.index(q)] < 1e29:
                dcurves[g][i] = curves[g][grid.index(q)]
            else:
                one = dict(label="curve", stages=[dict(groups=[g], quotas=[q], offsets=[0])])
                dcurves[g][i] = median_plan(one, 2)[0]
    try:
        dchosen, dpredicted = mb.plan_choose(deciles, dcurves, cus)
    except mb.MosaicError:
        dchosen, dpredicted = None, None          # no decile split fits every module

    plans = [packed(p, "named") for p in wl["plans"]]
    plans.append(packed(chosen, "chosen from the curves (Eq. 4-5)"))
    if dchosen is not None and dpredicted < 1e29:
        plans.append(dict(packed(dchosen, "chosen from curves on the decile grid (Sec. 3.4 granularity)"), predicted_ms=round(dpredicted, 4)))
    if ngroups == 3:
        # the two small modules share one quota and run back to back beside the large one
        big = max(range(ngroups), key=lambda g: group_ms_full[g])
        small = [g for g in range(ngroups) if g != big]
        best = None
        for qi, q in enumerate(grid):
            if (cus - q) not in grid:
                continue
            ts_ = [curves[g][qi] for g in small]
            tb = curves[big][grid.index(cus - q)]
            if max(ts_) < 1e29 and tb < 1e29:
                t = max(sum(ts_), tb)
                if best is None or t < best[0]:
                    best = (t, q)
        if best:
            q = best[1]
            qs, offs = [q] * ngroups, [cus - q] * ngroups
            qs[big], offs[big] = cus - q, 0
            plans.append(dict(label="small modules share a quota", predicted_ms=round(best[0], 4),
                              stages=[dict(groups=list(range(ngroups)), quotas=qs, offsets=offs)]))
    if ngroups >= 3:
        # Alg. 1 on the measured curves: stages of modules that pay to run side by side
        # (the planner takes up to 16 quota levels: the measured ones, thinned if need be, plus the whole device)
        lv = sorted({q for row in curves for q, v in zip(grid, row) if v < 1e29})
        while len(lv) > 15:
            lv = lv[::2] if lv[-1] == lv[::2][-1] else lv[::2] + [lv[-1]]
        full = [[row[grid.index(q)] if row[grid.index(q)] < 1e29 else 1e9 for q in lv] + [group_ms_full[g]] for g, row in enumerate(curves)]
        st_, alloc, t_pred, _ = mb.planner_solve(ngroups, [], lv + [cus], full, cus)
        if len(st_) > 1:
            stages = [dict(groups=list(members), quotas=[alloc[m] for m in members], offsets=pack([alloc[m] for m in members]))
                      for members in st_]
            plans.append(dict(label="planner stages (Alg. 1)", predicted_ms=round(t_pred, 4), stages=stages))
    if forced is not None:
        plans.append(packed(forced, "forced"))
    results, seen = [], set()
    for p in plans:
        key = json.dumps(p["stages"])
        if key in seen:
            continue
        seen.add(key)
        ms, pg = median_plan(p, 3)
        results.append(dict(p, iteration_ms=ms, group_ms=pg))
    best = min(results, key=lambda r: r["iteration_ms"])
    if forced is not None:
        best = [r for r in results if r["label"] == "forced"][0]

    # the timed region: K iterations under the best plan, inputs resident in HBM
    reserve(best)
    for _ in range(warmup):
        run_plan(best)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_plan(best)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    def util(fl, ms, q):
        return fl / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12 * q / cus)

    def quota_of(plan, g):
        for st in plan["stages"]:
            if g in st["groups"]:
                return st["quotas"][st["groups"].index(g)]

    out = {
        "workload": f"configs[{config}] {wl['name']}: " + ", ".join(
            f"{m['name']} B{m['batch']} N{m['seq']} h{m['hidden'] or m['out_dim']} L{m['layers']}" for m in wl["modules"]),
        "dtype": wl["dtype"], "batch": B, "groups": stage.groups, "total_tflop": round(sum(gflop) / 1e12, 3),
        "value": round(B / (ms_per_step * 1e-3), 2), "ms_per_step": round(ms_per_step, 4),
        "plan": dict(label=best["label"], stages=best["stages"]),
        "time_sliced": {"ms_per_step": round(ts_ms, 4), "samples_per_s": round(B / (ts_ms * 1e-3), 2),
                        "group_ms_at_all_cus": [round(v, 4) for v in group_ms_full],
                        "mfma_util": [round(util(gflop[g], group_ms_full[g], cus), 4) for g in range(ngroups)],
                        "aggregate_mfma_util": round(sum(gflop) / (ts_ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12), 4)},
        "colocated": {"speedup_vs_time_sliced": round(ts_ms / best["iteration_ms"], 4),
                      "speedup_vs_time_sliced_timed_region": round(ts_ms / ms_per_step, 4),
                      "group_ms_at_quota": [round(v, 4) for v in best["group_ms"]],
                      "mfma_util_at_quota": [round(util(gflop[g], best["group_ms"][g], quota_of(best, g)), 4) for g in range(ngroups)],
                      "aggregate_mfma_util": round(sum(gflop) / (best["iteration_ms"] * 1e-3) / (PEAK_BF16_TFLOPS * 1e12), 4),
                      "plans": [dict(label=r["label"], stages=[dict(groups=st["groups"], cus=st["quotas"], offsets=st["offsets"]) for st in r["stages"]],
                                     iteration_ms=round(r["iteration_ms"], 4), speedup_vs_time_sliced=round(ts_ms / r["iteration_ms"], 4),
                                     **({"predicted_ms": r["predicted_ms"]} if "predicted_ms" in r else {})) for r in results],
                      "chosen_from_curves": {"plan": chosen, "predicted_ms": round(predicted, 4), "cu_grid_step": 8,
                                             "group_ms": [{str(q): round(v, 4) for q, v in zip(grid, row) if v < 1e29} for row in curves]}},
    }
    if layer_split and ngroups >= 2:
        out["colocated"]["decoder_cut_in_time"] = decoder_cut(mb, synth, config, stage, results, group_ms_full, ts_ms)
    else:
        stage.destroy()
    mb.pool_clear()
    return out


def decoder_cut(mb, synth, config, stage, results, group_ms_full, ts_ms):
    """Two-stage alternative: the decoder cut after layer k, layers [0, k) colocated with the
    other groups, layers [k, L) alone on all CUs.  (plan, k) is picked from the colocated group
    times already measured (a decoder's time is linear in its layers), then measured."""
    from paper_2605_18710_amd.workload import SplitStage
    wl = synth.WORKLOADS[config]
    llm = [m for m in wl["modules"] if m["kind"] == "decoder"][0]
    L = llm["layers"]
    dec_g = [gi for gi, g in enumerate(stage.groups) if llm["name"] in g][0]
    cands = []
    for r in results:
        if len(r["stages"]) != 1 or len(set(r["stages"][0]["offsets"])) != len(r["stages"][0]["offsets"]):
            continue
        g_ms = r["group_ms"]
        others = max(v for gi, v in enumerate(g_ms) if gi != dec_g)
        for k in range(1, L):
            cands.append((max(others, g_ms[dec_g] * k / L) + group_ms_full[dec_g] * (L - k) / L, r["stages"][0]["quotas"], k))
    B = stage.batch
    stage.destroy()
    if not cands:
        return None
    pred, sp_plan, sp_k = min(cands)
    ss = SplitStage(config, sp_k, sp_plan)
    ss.run()
    rs = [ss.run() for _ in range(5)]
    it = statistics.median(r["iteration_ms"] for r in rs)
    out = {"cut_after_layer": sp_k, "plan_cus": sp_plan, "predicted_ms": round(pred, 4), "iteration_ms": round(it, 4),
           "stage_ms": [round(statistics.median(r["stage_ms"][j] for r in rs), 4) for j in range(2)],
           "samples_per_s": round(B / (it * 1e-3), 2), "speedup_vs_time_sliced": round(ts_ms / it, 4)}
    ss.destroy()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4,
                    help="index into the workload list (default 4: vision + audio + 7B-shaped decoder, the largest single-GPU workload)")
    ap.add_argument("--secondary", type=int, default=1, help="a second workload reported in the same line (-1: none)")
    ap.add_argument("--roofline-only", action="store_true")
    ap.add_argument("--attention-only", action="store_true", help="only the attention kernels at the decoder's shape (for rocprofv3)")
    ap.add_argument("--bandwidth-only", action="store_true", help="only the bandwidth-bound kernels at the decoder's shapes (for rocprofv3)")
    ap.add_argument("--power-only", action="store_true", help="board power and clock under the 7B-shaped GEMM: the three forms, constant inputs, and the vendor library as context")
    ap.add_argument("--library-only", action="store_true", help="context: the forward GEMM beside torch.matmul (vendor library) at six shapes")
    ap.add_argument("--plan", default=None, help="comma-separated CU quotas, one per group: time this plan instead of the best measured one "
                    "(under rocprofv3 the measured ranking of plans is distorted)")
    ap.add_argument("--module-only", default=None, metavar="NAME",
                    help="only steps of one module of the workload (e.g. llm, vit, audio), alone on all CUs: the kernel mix of a step, for rocprofv3 --stats")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--layer-split", action="store_true",
                    help="also measure the two-stage plan that cuts the decoder in time (built after the timed steps)")
    ap.add_argument("--no-pool-bench", action="store_true",
                    help="skip the create/destroy microbenchmark of masked streams (the profiler's queue interception does not survive it)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the stage is a single-GPU construct and this build holds no "
              "collectives; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_18710_amd import binding as mb, synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    mb.lib()
    wl = synth.WORKLOADS[args.config]
    llm = [m for m in wl["modules"] if m["kind"] == "decoder"][0]
    Tl, hl, fl = llm["batch"] * llm["seq"], llm["hidden"], llm["mlp"]
    cus = mb.device_cu_count()

    if args.module_only:
        print(json.dumps(module_steps(mb, synth, args.config, args.module_only, args.steps, args.warmup)))
        return
    if args.attention_only:
        print(json.dumps(attention_kernels(mb, llm["batch"], llm["seq"], llm["heads"], hl // llm["heads"], 1, reps=50)))
        return
    if args.power_only:
        print(json.dumps(power_probe(mb)))
        return
    if args.library_only:
        print(json.dumps(library_compare(mb)))
        return
    if args.bandwidth_only:
        # plus a plain device copy of known size, so that HBM byte counters of the same run can be scaled
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"shape": {"T": Tl, "h": hl, "f": fl}, "gbs": bandwidth_kernels(mb, Tl, hl, fl, reps=20)}))
        return
    big = Tl * hl * fl > 1e12                       # calls of several ms: fewer of them
    gflops, gms = roofline_gemm(mb, Tl, hl, 2 * fl, reps=20 if big else 50, settle_ms=40.0)
    if args.roofline_only:
        # a plain device copy of known size, so that HBM byte counters of the same run can
        # be scaled: 1 GiB read + 1 GiB written per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"kernel": "gemm_bf16_kernel", "shape": [Tl, hl, 2 * fl], "ms": gms,
                          "tflops": {k: gflops / v / 1e9 for k, v in gms.items()}}))
        return
    bw = bandwidth_kernels(mb, Tl, hl, fl, reps=20)
    attn = attention_kernels(mb, llm["batch"], llm["seq"], llm["heads"], hl // llm["heads"], 1, reps=20 if big else 50)
    pool = None if args.no_pool_bench else stream_pool_latency(mb, cus)
    torch.cuda.empty_cache()

    forced = [int(x) for x in args.plan.split(",")] if args.plan else None
    main_rec = measure_workload(mb, synth, args.config, args.steps, args.warmup, forced, args.layer_split)
    torch.cuda.empty_cache()
    second = None
    if args.secondary >= 0 and args.secondary != args.config and forced is None:
        second = measure_workload(mb, synth, args.secondary, args.steps, args.warmup)
        torch.cuda.empty_cache()

    dominant = max(gms, key=lambda k: gms[k])       # the slowest of the three forms bounds the step
    ngroups = len(main_rec["groups"])
    line = {
        "metric": "colocated stage samples/sec vs time-sliced at 1 GPU; per-module MFMA util @quota",
        "value": main_rec["value"], "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl["dtype"], "data": "synthetic",
        "config": {"workload": main_rec["workload"], "plan": main_rec["plan"], "groups": main_rec["groups"],
                   "total_tflop_per_step": main_rec["total_tflop"], "mode": "decoupled staged buffers; stages one after another, modules of a stage colocated"},
        "time_sliced": main_rec["time_sliced"],
        "colocated": main_rec["colocated"],
        "roofline": {"bound": "mfma", "kernel": f"gemm_bf16 {dominant} T={Tl} k={hl} n={2 * fl} (the decoder's gate/up projection)",
                     "achieved": round(gflops / gms[dominant] / 1e9, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gflops / gms[dominant] / 1e9 / PEAK_BF16_TFLOPS, 4),
                     "traffic": profiled_traffic(dominant, (Tl, hl, 2 * fl)),
                     "algorithmic_bytes": 2 * (Tl * hl + hl * 2 * fl + Tl * 2 * fl),
                     "avg_ms": {k: round(v, 4) for k, v in gms.items()},
                     "all_forms_tflops": {k: round(gflops / v / 1e9, 2) for k, v in gms.items()},
                     "hbm_kernels_gbs": bw, "hbm_peak_gbs": PEAK_HBM_GBS},
        "attention": attn,
        "stream_pool": pool,
        "secondary": second,
        "paper_context": "paper reports up to 1.31x per-iteration speedup on 32x H100-80GB (other hardware, other metric)",
    }
    # what creating the stage's streams on demand would add to every step (one per group)
    if pool is not None:
        pool["share_of_step_if_on_demand"] = round(ngroups * pool["on_demand_create_destroy_ms"] /
                                                   (main_rec["ms_per_step"] + ngroups * pool["on_demand_create_destroy_ms"]), 4)
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
