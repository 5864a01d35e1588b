"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-side logic (mask arithmetic, plan validation, quota choice,
descriptor validation, parameter layout) behaves as the header states."""
import os
import re

import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import binding as mb
from paper_2605_18710_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "mosaic.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(mosaic_[a-z0-9_]+)\s*\(", text))
    assert len(declared) > 40
    l = mb.lib()
    for name in declared:
        assert hasattr(l, name), f"{name} is declared in mosaic.h but not exported"
    assert declared == set(mb.SIGNATURES), declared ^ set(mb.SIGNATURES)


def bits(words):
    return [i for i in range(32 * len(words)) if (words[i // 32] >> (i % 32)) & 1]


def test_mask_striped_takes_same_share_of_every_xcd():
    w = mb.cu_mask_build(256, 8, 64, 32, mb.STRIPED)
    b = bits(w)
    assert b == list(range(32, 96))
    per_xcd = [sum(1 for i in b if i % 8 == x) for x in range(8)]
    assert per_xcd == [8] * 8


def test_mask_xcd_aligned_fills_whole_xcds():
    w = mb.cu_mask_build(256, 8, 64, 64, mb.XCD_ALIGNED)
    b = bits(w)
    assert len(b) == 64 and {i % 8 for i in b} == {2, 3}
    assert sorted({i // 8 for i in b}) == list(range(32))


def test_masks_of_a_partition_are_disjoint_and_cover():
    for layout, splits in ((mb.STRIPED, [(0, 26), (26, 51), (77, 179)]), (mb.XCD_ALIGNED, [(0, 64), (64, 192)])):
        seen = set()
        for off, q in splits:
            b = set(bits(mb.cu_mask_build(256, 8, q, off, layout)))
            assert len(b) == q and not (b & seen)
            seen |= b
        assert seen == set(range(256))


@pytest.mark.parametrize("args,status", [
    ((256, 8, 0, 0, mb.STRIPED), mb.EQUOTA),
    ((256, 8, 257, 0, mb.STRIPED), mb.EQUOTA),
    ((256, 8, 128, 192, mb.STRIPED), mb.EQUOTA),
    ((256, 8, 48, 0, mb.XCD_ALIGNED), mb.EQUOTA),
    ((256, 8, 64, 0, 7), mb.EINVAL),
    ((250, 8, 64, 0, mb.STRIPED), mb.EINVAL),
])
def test_mask_errors(args, status):
    with pytest.raises(mb.MosaicError) as e:
        mb.cu_mask_build(*args)
    assert e.value.status == status


def test_plan_validation_eq5():
    mb.plan_validate([64, 192], [0, 64], mb.STRIPED, mb.COLOCATED, 256, 8)
    mb.plan_validate([64, 64, 128], [0, 0, 64], mb.STRIPED, mb.COLOCATED, 256, 8)     # two modules share a stream
    mb.plan_validate([256, 256], [0, 0], mb.STRIPED, mb.TIME_SLICED, 256, 8)
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_validate([128, 192], [0, 64], mb.STRIPED, mb.COLOCATED, 256, 8)     # overlap
    assert e.value.status == mb.EQUOTA
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_validate([128, 192], [0, 128], mb.STRIPED, mb.COLOCATED, 256, 8)    # leaves the device
    assert e.value.status == mb.EQUOTA
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_validate([64, 0], [0, 64], mb.STRIPED, mb.COLOCATED, 256, 8)
    assert e.value.status == mb.EQUOTA
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_validate([64, 64], [0, 64], mb.STRIPED, 9, 256, 8)
    assert e.value.status == mb.EINVAL


def test_plan_needs_a_hardware_queue_per_stream(monkeypatch):
    """Streams that would have to share a hardware queue run one after the other: a colocated
    plan with more distinct streams than queues is refused, modules that share a quota count once."""
    monkeypatch.setenv("GPU_MAX_HW_QUEUES", "4")
    assert mb.device_hw_queues() == 4
    five = ([32, 32, 32, 32, 128], [0, 32, 64, 96, 128])
    assert mb.plan_stream_count(*five, mb.STRIPED, mb.COLOCATED) == 5
    assert mb.plan_stream_count(*five, mb.STRIPED, mb.TIME_SLICED) == 1
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_validate(*five, mb.STRIPED, mb.COLOCATED, 256, 8)
    assert e.value.status == mb.EQUOTA and "hardware queues" in str(e.value)
    shared = ([32, 32, 32, 32, 128], [0, 0, 32, 64, 96])          # the first two modules share a stream
    assert mb.plan_stream_count(*shared, mb.STRIPED, mb.COLOCATED) == 4
    mb.plan_validate(*shared, mb.STRIPED, mb.COLOCATED, 256, 8)
    monkeypatch.setenv("GPU_MAX_HW_QUEUES", "8")
    mb.plan_validate(*five, mb.STRIPED, mb.COLOCATED, 256, 8)


def test_plan_choose_matches_exhaustive_oracle():
    pts = [32, 64, 96, 128, 160, 192, 224]
    for seed in range(20):
        n_mod = 2 + seed % 2
        base = synth.uniform(900 + seed, (n_mod,), 1.0, 50.0)
        noise = synth.uniform(950 + seed, (n_mod, len(pts)), 0.9, 1.1)
        times = [[float(np.float32(base[m] * 256.0 / q * noise[m, i])) for i, q in enumerate(pts)] for m in range(n_mod)]
        q, t = mb.plan_choose(pts, times, 256)
        curves = [{pts[i]: times[m][i] for i in range(len(pts))} for m in range(n_mod)]
        q_ref, t_ref = O.best_split(curves, 256)
        assert q == q_ref and abs(t - t_ref) < 1e-6 * t_ref
        assert sum(q) <= 256
    with pytest.raises(mb.MosaicError) as e:
        mb.plan_choose([192, 224], [[1, 1], [1, 1]], 256)
    assert e.value.status == mb.EQUOTA


def _desc(**kw):
    base = dict(kind="decoder", layers=2, hidden=64, heads=4, mlp=96, batch=2, seq=16,
                norm="rmsnorm", act="swiglu", causal=1, bias=0, eps=1e-5)
    base.update(kw)
    return base


def _create(cfg, dtype="bf16"):
    import ctypes as C
    d = mb.make_desc(cfg, dtype)
    h = C.c_void_p()
    st = mb.lib().mosaic_module_create(C.byref(d), C.byref(h))
    return st, h


def test_module_descriptor_validation():
    import ctypes as C
    st, h = _create(_desc())
    assert st == mb.OK
    l = mb.lib()
    names = []
    buf = C.create_string_buffer(32)
    off, r, c = C.c_int64(), C.c_int64(), C.c_int64()
    total = 0
    for i in range(l.mosaic_module_tensor_count(h)):
        assert l.mosaic_module_tensor_info(h, i, buf, C.byref(off), C.byref(r), C.byref(c)) == mb.OK
        names.append(buf.value.decode())
        assert off.value == total and off.value % 8 == 0
        total += (r.value * c.value + 7) // 8 * 8
    assert names[:6] == ["L0.rms1_g", "L0.w_qkv", "L0.w_o", "L0.rms2_g", "L0.w_gu", "L0.w_down"]
    assert l.mosaic_module_param_bytes(h) == total * 2
    assert l.mosaic_module_workspace_bytes(h) > 0
    assert l.mosaic_module_input_elems(h) == 2 * 16 * 64
    assert l.mosaic_module_tensor_info(h, 99, buf, None, None, None) == mb.EINVAL
    l.mosaic_module_destroy(h)
    for bad, status in ((dict(hidden=66), mb.EINVAL),            # hidden % heads
                        (dict(hidden=1024, heads=4), mb.EUNSUPPORTED),   # head size 256
                        (dict(hidden=36, heads=4, mlp=96), mb.EUNSUPPORTED),   # not a multiple of 8
                        (dict(layers=0), mb.EINVAL), (dict(norm="none"), mb.EINVAL),
                        (dict(eps=0.0), mb.EINVAL), (dict(batch=0), mb.EINVAL)):
        st, _ = _create(_desc(**bad))
        assert st == status, bad
    st, _ = _create(dict(kind="projector", batch=2, seq=4, in_dim=0, out_dim=16))
    assert st == mb.EINVAL
    st, _ = _create(dict(kind="patch_stem", batch=2, seq=15, hidden=16, in_dim=12, patch=2))
    assert st == mb.EINVAL     # 15 is not a square grid
    st, _ = _create(dict(kind="text_stem", batch=2, seq=8, hidden=16, vocab=10, n_img=9))
    assert st == mb.EINVAL


def test_encoder_layout_has_biases_and_betas():
    import ctypes as C
    st, h = _create(dict(kind="encoder", layers=1, hidden=32, heads=2, mlp=64, batch=1, seq=4,
                         norm="layernorm", act="gelu", causal=0, bias=1, eps=1e-5), "f32")
    assert st == mb.OK
    l = mb.lib()
    buf = C.create_string_buffer(32)
    names = []
    for i in range(l.mosaic_module_tensor_count(h)):
        l.mosaic_module_tensor_info(h, i, buf, None, None, None)
        names.append(buf.value.decode())
    assert names == ["L0.ln1_g", "L0.ln1_b", "L0.w_qkv", "L0.b_qkv", "L0.w_o", "L0.b_o",
                     "L0.ln2_g", "L0.ln2_b", "L0.w_1", "L0.b_1", "L0.w_2", "L0.b_2"]
    l.mosaic_module_destroy(h)


def test_unbound_module_and_null_arguments_are_errors_not_crashes():
    import ctypes as C
    l = mb.lib()
    st, h = _create(_desc())
    assert l.mosaic_module_forward(h, 64, None, 1, 1) == mb.EINVAL          # not bound
    assert l.mosaic_module_bind(h, None, None, None, 0) == mb.EINVAL
    assert l.mosaic_module_bind_ids(h, 1) == mb.EINVAL                      # not a text stem
    assert l.mosaic_module_create(None, None) == mb.EINVAL
    assert l.mosaic_stage_run(None, None, None) == mb.EINVAL
    assert b"null" in l.mosaic_last_error()
    l.mosaic_module_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    """The stage is a single-GPU construct: asking bench.py for more exits with a message."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_committed_gemm_traffic_parses_and_is_not_below_the_algorithmic_bytes():
    """bench.py's roofline.traffic comes from the committed counter summary: every form must
    parse, and HBM-side bytes cannot be below reading each operand and writing the output once."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    for (T, k, n) in bench.PROFILE_OF_SHAPE:         # the roofline shapes of configs[1] and of the 7B-shaped decoders
        if not os.path.exists(os.path.join(root, "profiles", bench.PROFILE_OF_SHAPE[(T, k, n)])):
            continue
        algorithmic = 2 * (T * k + k * n + T * n)
        for form in ("fprop", "dgrad", "wgrad"):
            t = bench.profiled_traffic(form, (T, k, n))
            assert isinstance(t, int) and algorithmic <= t < 8 * algorithmic, (form, t)
    assert bench.profiled_traffic("fprop", (8, 8, 8)) is None


def test_measured_step_bytes_cover_the_benchmarked_modules_and_are_not_below_the_model():
    """The counter-based utilisation proxy of the planner reads a committed table: every module
    of the two benchmarked workloads has a row, and no row claims fewer bytes than the
    algorithmic count (every operand read once, every result written once)."""
    from paper_2605_18710_amd import planning, synth
    table = planning.measured_step_bytes()
    assert table, "profiles/module_step_hbm_bytes.txt is missing or empty"
    for config in (4, 1):
        for m in synth.WORKLOADS[config]["modules"]:
            key = planning.shape_signature(m)
            assert key in table, key
            assert table[key] >= synth.module_bytes(m, 2), key
            assert table[key] <= 8.0 * synth.module_bytes(m, 2), key     # a re-read factor beyond this would be a parsing slip
    assert planning.measured_step_bytes("/nonexistent/table.txt") == {}


@pytest.mark.parametrize("T,k,n,pieces,cut_tiles,why", [
    (32768, 4096, 22016, 5, 96, "1376 tiles: the 96 past five rounds of 256, in 5 pieces"),
    (32768, 11008, 4096, 4, 176, "688 tiles: the 176 past two rounds, in 4 pieces"),
    (32768, 4096, 12288, 1, 0, "768 tiles: three whole rounds, nothing to cut"),
    (8192, 2048, 11264, 1, 0, "352 tiles but only 8192 tokens: pieces would be mostly fill and drain"),
    (8192, 2048, 2048, 4, 64, "64 tiles: all of them, in 256 / 64 pieces"),
    (4608, 1024, 1024, 8, 16, "16 tiles: all of them, in at most 8 pieces"),
    (1568, 768, 768, 1, 0, "9 tiles, 1568 tokens: too short to cut"),
])
def test_weight_gradient_split_is_a_function_of_the_shape(T, k, n, pieces, cut_tiles, why):
    """Which tiles of a weight gradient are cut along the token dimension, and into how many pieces,
    is decided by (T, k, n) alone (never the quota: the bits must not depend on it).  The scratch a
    caller must provide makes the decision visible: fp32 pieces of whole 256x256 tiles, then the
    partial column sums of the bias gradient."""
    got = mb.linear_wgrad_scratch_bytes(T, k, n)
    pieces_bytes = pieces * cut_tiles * 256 * 256 * 4 if pieces > 1 else 0
    aligned = (pieces_bytes + 255) // 256 * 256
    assert got == aligned + mb.colsum_scratch_bytes(n), why
