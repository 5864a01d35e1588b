"""Launcher tests on the GPU: CU masks confine work, the pool removes stream creation
from the stage path, and colocated / time-sliced execution give identical bits."""
import numpy as np
import pytest

from paper_2605_18710_amd import synth
from helpers import quantize, quantize_tree, to_dev, layer_params, load_layer_params

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_18710_amd import binding
    binding.lib()
    return binding


def test_device_shape(mb):
    assert mb.device_cu_count() == 256
    assert mb.device_xcd_count() == 8


def placement(mb, stream, n=2048):
    out = torch.full((n, 3), -1, dtype=torch.int32, device="cuda")
    mb.probe_placement(stream, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_masks_confine_workgroups(mb):
    full = placement(mb, None)
    all_cus = {tuple(r) for r in full}
    assert len({r[0] for r in full}) == 8            # eight XCDs seen without a mask
    # one queue spans all XCDs: a mask that empties an XCD is refused before HIP sees it
    with pytest.raises(mb.MosaicError) as e:
        mb.Stream(64, 64, mb.XCD_ALIGNED)
    assert e.value.status == mb.EUNSUPPORTED
    with pytest.raises(mb.MosaicError) as e:
        mb.Stream(4, 0, mb.STRIPED)
    assert e.value.status == mb.EQUOTA
    s_st = mb.Stream(64, 0, mb.STRIPED)
    got2 = placement(mb, s_st)
    cus2 = {tuple(r) for r in got2}
    assert len(cus2) <= 64 and len({r[0] for r in got2}) == 8
    per_xcd = [len({tuple(r) for r in got2 if r[0] == x}) for x in range(8)]
    assert max(per_xcd) <= 8
    s_b = mb.Stream(192, 64, mb.STRIPED)
    cus3 = {tuple(r) for r in placement(mb, s_b, 8192)}
    assert not (cus2 & cus3), "disjoint quotas landed on a common CU"
    assert len(all_cus) <= 256
    s_c = mb.Stream(8, 0, mb.STRIPED)          # smallest legal quota: one CU per XCD
    cus4 = {tuple(r) for r in placement(mb, s_c, 512)}
    assert len(cus4) <= 8 and len({c[0] for c in cus4}) == 8
    for s in (s_st, s_b, s_c):
        s.destroy()


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy().copy()


def test_stage_modes_agree_and_pool_is_used(mb):
    dtype = "bf16"
    cfgs = [dict(kind="encoder", batch=2, seq=196, hidden=256, heads=4, mlp=1024, layers=2, norm="layernorm",
                 act="gelu", causal=0, bias=1, eps=1e-5),
            dict(kind="decoder", batch=2, seq=256, hidden=512, heads=4, mlp=768, layers=2, norm="rmsnorm",
                 act="swiglu", causal=1, bias=0, eps=1e-5)]
    mods, xs, ys, dxs, tg, losses = [], [], [], [], [], []
    for i, cfg in enumerate(cfgs):
        m = mb.Module(cfg, dtype)
        load_layer_params(m, quantize_tree([layer_params(cfg, 5000 + 1000 * i + 100 * l) for l in range(cfg["layers"])], dtype))
        T, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
        mods.append(m)
        xs.append(to_dev(quantize(synth.normal(6000 + i, (T, h)), dtype), dtype))
        tg.append(to_dev(quantize(synth.normal(6100 + i, (T, h)), dtype), dtype))
        ys.append(torch.empty_like(xs[-1])); dxs.append(torch.empty_like(xs[-1]))
        losses.append(torch.zeros(1, dtype=torch.float32, device="cuda"))
    with pytest.raises(mb.MosaicError) as e:      # nothing reserved yet for this split
        mb.stage_run(mods, xs, ys, [40, 216], [0, 40], mb.STRIPED, mb.COLOCATED, target=tg, dx=dxs, loss=losses)
    assert e.value.status == mb.EQUOTA
    for q, o, lay in ((256, 0, mb.STRIPED), (64, 0, mb.STRIPED), (192, 64, mb.STRIPED), (128, 0, mb.STRIPED), (128, 128, mb.STRIPED)):
        mb.pool_reserve(q, o, lay)
    created = mb.pool_creations()
    snaps = []
    runs = [([256, 256], [0, 0], mb.STRIPED, mb.TIME_SLICED), ([64, 192], [0, 64], mb.STRIPED, mb.COLOCATED),
            ([128, 128], [0, 128], mb.STRIPED, mb.COLOCATED)]
    for quotas, offs, lay, mode in runs:
        for m in mods:
            m.grads.zero_()
        r = mb.stage_run(mods, xs, ys, quotas, offs, lay, mode, target=tg, dx=dxs, loss=losses)
        assert r["stage_ms"] > 0 and all(t > 0 for t in r["module_ms"])
        if mode == mb.TIME_SLICED:
            assert r["stage_ms"] >= sum(r["module_ms"]) * 0.999          # Eq. 1
        else:
            assert r["stage_ms"] >= max(r["module_ms"]) * 0.999          # Eq. 4
        snaps.append([bits(t) for t in ys + dxs + losses] + [bits(m.grads) for m in mods])
    assert mb.pool_creations() == created, "a stream was created on the stage path"
    for s in snaps[1:]:
        for a, b in zip(s, snaps[0]):
            assert np.array_equal(a, b), "colocated and time-sliced runs differ"
    with pytest.raises(mb.MosaicError) as e:
        mb.stage_run(mods, xs, ys, [128, 192], [0, 64], mb.STRIPED, mb.COLOCATED, target=tg, dx=dxs, loss=losses)
    assert e.value.status == mb.EQUOTA
    for m in mods:
        m.destroy()


def test_decoder_cut_in_time_runs_two_stages(mb):
    """Two-stage plan: layers [0, k) of the decoder colocated with the vision group, layers
    [k, L) alone on all CUs.  Both stages must run, and the iteration is their sum (Eq. 1)."""
    from paper_2605_18710_amd.workload import SplitStage
    with pytest.raises(ValueError):
        SplitStage(0, 1)                        # the tiny workload's decoder has one layer: nothing to cut
    st = SplitStage(1, 2, [32, 224])
    try:
        created = mb.pool_creations()
        st.run()
        r = st.run()
        assert mb.pool_creations() == created, "an iteration created a stream"
        assert len(r["stage_ms"]) == 2 and all(t > 0 for t in r["stage_ms"])
        # the iteration is timed by the host clock across both stages: at least their sum (Eq. 1),
        # and not much more (the gap between the two calls)
        assert sum(r["stage_ms"]) <= r["iteration_ms"] <= sum(r["stage_ms"]) + 5.0
        assert len(r["module_ms"]) == len(st.first) + 1
        for m in st.first + [st.second]:
            assert torch.isfinite(m.y.float()).all()
        assert torch.isfinite(st.second.loss).all() and float(st.second.loss) > 0
    finally:
        st.destroy()
        mb.pool_clear()
