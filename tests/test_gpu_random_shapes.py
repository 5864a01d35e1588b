"""Seeded random shapes: linear, attention (with grouped key/value heads) and norm kernels
against the CPU checker, each at two quotas drawn from the 8-CU grid, bit-identical between
them.  The shapes are drawn from a fixed seed, so the run is reproducible."""
import random

import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import rel_l2, quantize, to_dev, from_dev, assert_close

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
QS = [256, 224, 192, 160, 128, 96, 64, 40, 32, 24, 8]


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_18710_amd import binding
    binding.lib()
    return binding


def empty(shape):
    return torch.empty(shape, dtype=torch.bfloat16, device="cuda")


def bits(t):
    return t.view(torch.int16).cpu().numpy().copy()


def test_random_linear_shapes(mb):
    rng = random.Random(18710)
    for it in range(16):
        T = rng.choice([8, 40, 100, 257, 600, 1000, 1568, 2100]) + 8 * rng.randrange(0, 4)
        k = 8 * rng.randrange(1, 100); n = 8 * rng.randrange(1, 100)
        use_b, use_r = rng.random() < 0.5, rng.random() < 0.5
        X = quantize(synth.normal(100 + it, (T, k)), "bf16"); W = quantize(synth.normal(200 + it, (k, n), 0, 0.05), "bf16")
        b = quantize(synth.normal(300 + it, (n,), 0, 0.1), "bf16"); R = quantize(synth.normal(400 + it, (T, n)), "bf16")
        dY = quantize(synth.normal(500 + it, (T, n)), "bf16")
        X_, W_, b_, R_, dY_ = [to_dev(a, "bf16") for a in (X, W, b, R, dY)]
        ref_y = O.linear_fwd(X, W, b if use_b else None) + (R if use_r else 0)
        ref_dx, ref_dw, _ = O.linear_bwd(X, W, dY)
        outs = []
        for q in rng.sample(QS, 2):
            Y = empty((T, n)); dX = empty((T, k)); dW = empty((k, n)); db = empty((n,))
            sc = torch.empty(max(16, mb.linear_wgrad_scratch_bytes(T, k, n)), dtype=torch.uint8, device="cuda")
            mb.op_linear_fwd(None, q, "bf16", T, k, n, X_, W_, b_ if use_b else None, R_ if use_r else None, Y)
            mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, None, dX)
            mb.op_linear_wgrad(None, q, "bf16", T, k, n, X_, dY_, dW, db if use_b else None, sc)
            torch.cuda.synchronize()
            outs.append([bits(t) for t in (Y, dX, dW)])
        info = (T, k, n, use_b, use_r)
        assert_close(from_dev(Y), ref_y, "bf16", ("Y",) + info)
        assert_close(from_dev(dX), ref_dx, "bf16", ("dX",) + info)
        assert_close(from_dev(dW), ref_dw, "bf16", ("dW",) + info)
        assert all(np.array_equal(a, b0) for a, b0 in zip(outs[0], outs[1])), info


def test_random_input_gradient_shapes_with_contractions_of_whole_128s(mb):
    """The input gradient has a kernel of its own for contractions that are a multiple of 128
    long; which tiles it computes depends on the quota.  Random output shapes (ragged in both
    dimensions), with and without the residual, four quotas each including tiny ones: every
    element against the CPU checker, bits identical across the quotas."""
    rng = random.Random(4242)
    for it in range(12):
        T = rng.choice([8, 100, 257, 600, 1000, 1568, 2100, 4096]) + 8 * rng.randrange(0, 4)
        k = 8 * rng.randrange(1, 160); n = 128 * rng.randrange(1, 24)
        use_r = rng.random() < 0.5
        W = quantize(synth.normal(200 + it, (k, n), 0, 0.05), "bf16"); dY = quantize(synth.normal(500 + it, (T, n)), "bf16")
        R = quantize(synth.normal(400 + it, (T, k)), "bf16")
        W_, dY_, R_ = [to_dev(a, "bf16") for a in (W, dY, R)]
        ref_dx, _, _ = O.linear_bwd(np.zeros((T, k)), W, dY)
        if use_r:
            ref_dx = ref_dx + R
        outs = []
        for q in rng.sample(QS + [3, 1], 4):
            dX = empty((T, k))
            mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, R_ if use_r else None, dX)
            torch.cuda.synchronize()
            outs.append(bits(dX))
        info = (T, k, n, use_r)
        got = from_dev(dX)
        assert rel_l2(got, ref_dx) <= 2e-2, info
        # one bf16 rounding of an fp32 sum of n products of N(0,1) and N(0,0.05^2) values
        assert np.all(np.abs(got - ref_dx) <= 2.0 ** -7 * np.abs(ref_dx) + 1e-2 * np.sqrt(n) * 0.05), info
        assert all(np.array_equal(o, outs[0]) for o in outs[1:]), info


def test_random_attention_shapes(mb):
    rng = random.Random(18711)
    for it in range(12):
        d = rng.choice([64, 128, 128, 32]); Hkv = rng.choice([1, 2, 3]); H = Hkv * rng.choice([1, 1, 2, 4])
        B = rng.choice([1, 2, 3]); N = rng.choice([1, 31, 64, 100, 129, 200, 333, 512, 777]); causal = rng.choice([0, 1])
        width = (H + 2 * Hkv) * d
        qkv = quantize(synth.normal(600 + it, (B * N, width)), "bf16"); dO = quantize(synth.normal(700 + it, (B * N, H * d)), "bf16")
        ref_o = O.attention_fwd(qkv, B, N, H, causal, Hkv); ref_d = O.attention_bwd(qkv, dO, B, N, H, causal, Hkv)
        qkv_, dO_ = to_dev(qkv, "bf16"), to_dev(dO, "bf16")
        outs = []
        for q in rng.sample(QS, 2):
            Oo = empty((B * N, H * d)); lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
            dq = empty((B * N, width)); delta = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
            mb.op_attention_gqa_fwd(None, q, "bf16", B, N, H, Hkv, d, causal, qkv_, Oo, lse)
            mb.op_attention_gqa_bwd(None, q, "bf16", B, N, H, Hkv, d, causal, qkv_, Oo, lse, dO_, dq, delta)
            torch.cuda.synchronize()
            outs.append([bits(Oo), bits(dq)])
        info = (B, N, H, Hkv, d, causal)
        assert_close(from_dev(Oo), ref_o, "bf16", ("O",) + info, roundings=2)
        assert_close(from_dev(dq), ref_d, "bf16", ("dqkv",) + info, roundings=8)
        assert all(np.array_equal(a, b0) for a, b0 in zip(outs[0], outs[1])), info


def test_random_norm_shapes(mb):
    rng = random.Random(18712)
    for it in range(10):
        norm = rng.choice(["layernorm", "rmsnorm"]); h = 8 * rng.choice([16, 96, 128, 160, 256, 400, 512, 640]); T = rng.choice([3, 50, 130, 999, 4100])
        x = quantize(synth.normal(800 + it, (T, h)), "bf16"); g = quantize(1 + synth.normal(820 + it, (h,), 0, 0.1), "bf16")
        be = quantize(synth.normal(840 + it, (h,), 0, 0.1), "bf16")
        dy = quantize(synth.normal(860 + it, (T, h)), "bf16"); R = quantize(synth.normal(880 + it, (T, h)), "bf16")
        ln = norm == "layernorm"
        y_ref = O.layernorm_fwd(x, g, be, 1e-5) if ln else O.rmsnorm_fwd(x, g, 1e-5)
        x_, g_, be_, dy_, R_ = [to_dev(a, "bf16") for a in (x, g, be, dy, R)]
        outs = []
        for q in rng.sample(QS, 2):
            y = empty((T, h)); st = torch.empty((T, 2), dtype=torch.float32, device="cuda"); dx = empty((T, h)); dg = empty((h,)); db = empty((h,))
            sc = torch.empty(mb.norm_bwd_scratch_bytes(h), dtype=torch.uint8, device="cuda")
            mb.op_norm_fwd(None, q, "bf16", norm, T, h, 1e-5, x_, g_, be_ if ln else None, y, st)
            mb.op_norm_bwd(None, q, "bf16", norm, T, h, x_, g_, st, dy_, R_, dx, dg, db if ln else None, sc)
            torch.cuda.synchronize()
            outs.append([bits(y), bits(dx), bits(dg)])
        res = O.layernorm_bwd(x, g, dy, 1e-5) if ln else O.rmsnorm_bwd(x, g, dy, 1e-5)
        info = (norm, T, h)
        assert_close(from_dev(y), y_ref, "bf16", ("y",) + info)
        assert_close(from_dev(dx), res[0] + R, "bf16", ("dx",) + info, roundings=2)
        assert_close(from_dev(dg), res[1], "bf16", ("dgamma",) + info, roundings=2)
        assert all(np.array_equal(a, b0) for a, b0 in zip(outs[0], outs[1])), info
