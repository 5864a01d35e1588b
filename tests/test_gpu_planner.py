"""GPU test of the planned execution of a job with a real parallel-encoder stage: a
CLIP-like DAG (vision encoder || text encoder, each followed by its projection head).
The planner's stages are executed one after another, each colocated under its quotas, and
every module's output and gradients must equal, bit for bit, what the same module
produces alone on the whole device."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mb():
    from paper_2605_18710_amd import binding
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    binding.lib()
    return binding


def test_clip_like_job_is_planned_and_run(mb):
    from paper_2605_18710_amd import synth
    from paper_2605_18710_amd.planning import PlannedJob
    mods = [synth._enc("vision", 4, 196, 256, 4, 1024, 2), synth._enc("text", 4, 128, 256, 4, 1024, 2),
            synth._proj("vproj", 4, 196, 256, 256), synth._proj("tproj", 4, 128, 256, 256)]
    job = PlannedJob(mods, [("vision", "vproj"), ("text", "tproj")], "bf16")
    try:
        grid = [32, 64, 128, 192, 256]
        times = job.measure_curves(grid, iters=2)
        assert all(t > 0 for row in times for t in row)
        bw = job.bandwidth_table(times)
        assert all(0.0 <= b <= 1.0 for row in bw for b in row)
        # shapes nobody profiled: the counter-based table falls back to the algorithmic bytes
        assert job.bandwidth_table(times, proxy="counters") == bw
        with pytest.raises(ValueError):
            job.bandwidth_table(times, proxy="nonsense")
        fit = job.fit_interference(grid, times, bw, [{0: 128, 1: 128}, {0: 64, 1: 192}, {0: 192, 1: 64}, {2: 128, 3: 128},
                                                      {0: 32, 1: 192}, {2: 64, 3: 192}], iters=2)
        assert fit["n_obs"] == 12 and np.isfinite(fit["r2"]) and fit["r2"] >= fit["r2_additive"] - 1e-9
        stages, alloc, t_iter, stats = job.solve(grid, times)
        where = {m: i for i, st in enumerate(stages) for m in st}
        assert sorted(where) == [0, 1, 2, 3]
        assert where[0] < where[2] and where[1] < where[3]
        for st in stages:
            assert sum(alloc[m] for m in st) <= 256
        # reference: every module alone on the whole device
        ref = []
        for m in range(4):
            job._run([m], [256], 1)
            s = job.staged[m]
            ref.append((s.y.clone(), s.dx.clone(), s.module.grads.clone()))
            s.y.zero_(); s.dx.zero_(); s.module.grads.zero_()
        res = job.run_plan(stages, alloc, iters=2)
        assert res["iteration_ms"] > 0 and len(res["stage_ms"]) == len(stages)
        for m in range(4):
            s = job.staged[m]
            for got, want in zip((s.y, s.dx, s.module.grads), ref[m]):
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (m,)
    finally:
        job.destroy()
