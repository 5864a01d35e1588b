"""Pins for the layer variants of the CPU checker (tanh GELU, rotary position embedding,
AdamW): closed forms, invariants, finite differences, and the same quantities computed
by an independent library routine (PyTorch on the CPU)."""
import numpy as np
import pytest
import torch

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import layer_params, small_cfg


# ---------------------------------------------------------------------- tanh GELU
def test_gelu_tanh_special_values_and_library():
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert O.gelu_tanh_grad(np.array([0.0]))[0] == 0.5
    z = synth.normal(9001, (257,), 0.0, 2.0)
    assert np.allclose(O.gelu_tanh(-z), O.gelu_tanh(z) - z, atol=1e-15)          # odd part is z/2
    assert np.allclose(O.gelu_tanh(np.array([12.0])), 12.0, atol=1e-12)
    ref = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    assert np.allclose(O.gelu_tanh(z), ref, rtol=0, atol=1e-14)
    # it is an approximation of the erf form: close, not equal
    assert 1e-5 < np.abs(O.gelu_tanh(z) - O.gelu(z)).max() < 1e-3


def test_gelu_tanh_grad_by_finite_differences():
    z = synth.normal(9002, (101,), 0.0, 1.5)
    fd = (O.gelu_tanh(z + 1e-6) - O.gelu_tanh(z - 1e-6)) / 2e-6
    assert np.allclose(O.gelu_tanh_grad(z), fd, atol=1e-8)


# ---------------------------------------------------------------------------- RoPE
def test_rope_is_a_rotation_identity_at_position_zero_and_leaves_v():
    B, N, H, d = 2, 9, 3, 8
    h = H * d
    qkv = synth.normal(9010, (B * N, 3 * h))
    r = O.rope_rotate(qkv, B, N, H, 10000.0)
    assert np.array_equal(r[:, 2 * h:], qkv[:, 2 * h:])
    assert np.array_equal(r[0::N], qkv[0::N])                                   # position 0 of every sample
    pairs = lambda a: a[:, :2 * h].reshape(B * N, 2 * H * d // 2, 2)
    assert np.allclose((pairs(r) ** 2).sum(-1), (pairs(qkv) ** 2).sum(-1), atol=1e-13)   # each pair keeps its length
    back = O.rope_rotate(r, B, N, H, 10000.0, -1.0)
    assert np.allclose(back, qkv, atol=1e-13)                                   # transpose = inverse
    assert not np.allclose(r[1::N, :2 * h], qkv[1::N, :2 * h])


def test_rope_pair_angles_written_out():
    # one head of size 4 at position 3: pair 0 turns by 3 rad, pair 1 by 3 * base^(-1/2)
    base = 100.0
    qkv = np.zeros((4, 12)); qkv[3, 0:4] = [1.0, 0.0, 0.0, 2.0]; qkv[3, 4:8] = [0.0, 1.0, 1.0, 0.0]
    r = O.rope_rotate(qkv, 1, 4, 1, base)
    a0, a1 = 3.0, 3.0 / 10.0
    assert np.allclose(r[3, 0:4], [np.cos(a0), np.sin(a0), -2.0 * np.sin(a1), 2.0 * np.cos(a1)], atol=1e-15)
    assert np.allclose(r[3, 4:8], [-np.sin(a0), np.cos(a0), np.cos(a1), np.sin(a1)], atol=1e-15)


def test_rope_scores_depend_on_relative_position_only():
    # the same q and k vectors placed at (m, n) and at (m + s, n + s) give the same dot product
    H, d, N = 1, 16, 12
    qv, kv = synth.normal(9011, (d,)), synth.normal(9012, (d,))
    def score(m, n):
        qkv = np.zeros((N, 3 * d)); qkv[m, :d] = qv; qkv[n, d:2 * d] = kv
        r = O.rope_rotate(qkv, 1, N, H, 10000.0)
        return float(r[m, :d] @ r[n, d:2 * d])
    assert score(5, 2) == pytest.approx(score(9, 6), abs=1e-12)
    assert score(5, 2) != pytest.approx(score(5, 3), abs=1e-6)


def test_decoder_layer_with_rope_by_finite_differences():
    cfg = dict(small_cfg("decoder"), rope=100.0)
    p = {k: v * (10.0 if v.ndim == 2 else 1.0) for k, v in layer_params(cfg, 9020).items()}
    x = synth.normal(9021, (cfg["batch"] * cfg["seq"], cfg["hidden"]))
    R = synth.normal(9022, x.shape)
    y, s = O.layer_fwd(x, p, cfg)
    dx, g = O.layer_bwd(R, p, s, cfg)
    y0, _ = O.layer_fwd(x, p, dict(cfg, rope=0))
    assert np.abs(y - y0).max() > 1e-4                                          # the option does something
    loss = lambda pp, xx=x: float((O.layer_fwd(xx, pp, cfg)[0] * R).sum())
    for key in p:
        D = synth.normal(9030 + len(key), p[key].shape)
        pp, pm = dict(p), dict(p)
        pp[key] = p[key] + 1e-5 * D; pm[key] = p[key] - 1e-5 * D
        fd = (loss(pp) - loss(pm)) / 2e-5
        assert fd == pytest.approx(float((g[key] * D).sum()), rel=1e-6, abs=1e-9), key
    D = synth.normal(9040, x.shape)
    fd = (loss(p, x + 1e-5 * D) - loss(p, x - 1e-5 * D)) / 2e-5
    assert fd == pytest.approx(float((dx * D).sum()), rel=1e-6, abs=1e-9)


def test_encoder_layer_with_tanh_gelu_by_finite_differences():
    cfg = dict(small_cfg("encoder"), act="gelu_tanh")
    p = {k: v * (10.0 if v.ndim == 2 else 1.0) for k, v in layer_params(cfg, 9050).items()}
    x = synth.normal(9051, (cfg["batch"] * cfg["seq"], cfg["hidden"]))
    R = synth.normal(9052, x.shape)
    y, s = O.layer_fwd(x, p, cfg)
    _, g = O.layer_bwd(R, p, s, cfg)
    loss = lambda pp: float((O.layer_fwd(x, pp, cfg)[0] * R).sum())
    for key in ("w_1", "b_1", "w_2"):
        D = synth.normal(9060 + len(key), p[key].shape)
        pp, pm = dict(p), dict(p)
        pp[key] = p[key] + 1e-5 * D; pm[key] = p[key] - 1e-5 * D
        assert (loss(pp) - loss(pm)) / 2e-5 == pytest.approx(float((g[key] * D).sum()), rel=1e-6, abs=1e-9), key


# ------------------------------------------------------------ grouped-query attention
def test_gqa_equals_mha_with_repeated_kv_heads():
    # sharing a K/V head inside a group is the same as giving every query head its own copy;
    # the shared head's gradient is the sum of the copies' gradients
    B, N, H, Hkv, d = 2, 7, 6, 2, 4
    G = H // Hkv
    qkv = synth.normal(9200, (B * N, (H + 2 * Hkv) * d))
    do = synth.normal(9201, (B * N, H * d))
    q, k, v = qkv[:, :H * d], qkv[:, H * d:(H + Hkv) * d], qkv[:, (H + Hkv) * d:]
    rep = lambda a: np.concatenate([a[:, (t // G) * d:(t // G + 1) * d] for t in range(H)], axis=1)
    full = np.concatenate([q, rep(k), rep(v)], axis=1)
    for causal in (0, 1):
        assert np.allclose(O.attention_fwd(qkv, B, N, H, causal, Hkv), O.attention_fwd(full, B, N, H, causal), atol=1e-14)
        assert np.allclose(O.attention_lse(qkv, B, N, H, causal, Hkv), O.attention_lse(full, B, N, H, causal), atol=1e-14)
        g, gf = O.attention_bwd(qkv, do, B, N, H, causal, Hkv), O.attention_bwd(full, do, B, N, H, causal)
        assert np.allclose(g[:, :H * d], gf[:, :H * d], atol=1e-14)
        for part, off_f in ((0, H * d), (1, 2 * H * d)):
            for u in range(Hkv):
                want = sum(gf[:, off_f + t * d:off_f + (t + 1) * d] for t in range(u * G, (u + 1) * G))
                c0 = (H + part * Hkv + u) * d
                assert np.allclose(g[:, c0:c0 + d], want, atol=1e-13)


def test_decoder_layer_with_gqa_and_rope_by_finite_differences():
    cfg = dict(small_cfg("decoder", h=16, H=4), kv_heads=2, rope=100.0)
    h, d = 16, 4
    p = {k: v * (10.0 if v.ndim == 2 else 1.0) for k, v in layer_params(cfg, 9220).items()}
    p["w_qkv"] = p["w_qkv"][:, :(4 + 2 * 2) * d].copy()
    x = synth.normal(9221, (cfg["batch"] * cfg["seq"], h))
    R = synth.normal(9222, x.shape)
    y, s = O.layer_fwd(x, p, cfg)
    dx, g = O.layer_bwd(R, p, s, cfg)
    assert g["w_qkv"].shape == p["w_qkv"].shape
    loss = lambda pp, xx=x: float((O.layer_fwd(xx, pp, cfg)[0] * R).sum())
    for key in ("w_qkv", "w_o", "rms1_g"):
        D = synth.normal(9230 + len(key), p[key].shape)
        pp, pm = dict(p), dict(p)
        pp[key] = p[key] + 1e-5 * D; pm[key] = p[key] - 1e-5 * D
        assert (loss(pp) - loss(pm)) / 2e-5 == pytest.approx(float((g[key] * D).sum()), rel=1e-6, abs=1e-9), key
    D = synth.normal(9240, x.shape)
    assert (loss(p, x + 1e-5 * D) - loss(p, x - 1e-5 * D)) / 2e-5 == pytest.approx(float((dx * D).sum()), rel=1e-6, abs=1e-9)


# ----------------------------------------------------------- strided-convolution stem
@pytest.mark.parametrize("stride,L", [(1, 9), (2, 10), (2, 7)])
def test_conv1d_matches_library_and_finite_differences(stride, L):
    B, C, Co = 2, 3, 5
    x = synth.normal(9300, (B, L, C)); w = synth.normal(9301, (3 * C, Co)); b = synth.normal(9302, (Co,))
    y = O.conv1d_fwd(x, w, b, stride)
    wt = torch.from_numpy(w.reshape(3, C, Co).transpose(2, 1, 0).copy())          # [Co, C, tap]
    ref = torch.nn.functional.conv1d(torch.from_numpy(x.transpose(0, 2, 1).copy()), wt, torch.from_numpy(b), stride=stride, padding=1)
    assert np.allclose(y, ref.numpy().transpose(0, 2, 1), atol=1e-13)
    R = synth.normal(9303, y.shape)
    dx, dw, db = O.conv1d_bwd(x, w, R, stride)
    for arr, grad, seed in ((x, dx, 1), (w, dw, 2), (b, db, 3)):
        D = synth.normal(9310 + seed, arr.shape)
        f = lambda e: float((O.conv1d_fwd(x + e * D if arr is x else x, w + e * D if arr is w else w, b + e * D if arr is b else b, stride) * R).sum())
        assert (f(1e-6) - f(-1e-6)) / 2e-6 == pytest.approx(float((grad * D).sum()), rel=1e-7, abs=1e-8)


def test_conv1d_border_taps_written_out():
    # one channel, identity-like taps: w = [1, 10, 100] picks x[t-1] + 10 x[t] + 100 x[t+1]
    x = np.arange(1.0, 6.0).reshape(1, 5, 1)
    w = np.array([[1.0], [10.0], [100.0]])
    y1 = O.conv1d_fwd(x, w, np.zeros(1), 1)[0, :, 0]
    assert np.array_equal(y1, [210.0, 321.0, 432.0, 543.0, 54.0])
    y2 = O.conv1d_fwd(x, w, np.zeros(1), 2)[0, :, 0]
    assert np.array_equal(y2, [210.0, 432.0, 54.0])                                  # frames 0, 2, 4


def test_conv_stem_by_finite_differences():
    B, N, C, h = 2, 5, 4, 6
    p = dict(w_c1=synth.normal(9320, (3 * C, h), 0, 0.3), b_c1=synth.normal(9321, (h,), 0, 0.1),
             w_c2=synth.normal(9322, (3 * h, h), 0, 0.3), b_c2=synth.normal(9323, (h,), 0, 0.1),
             pos=synth.normal(9324, (N, h), 0, 0.1))
    x = synth.normal(9325, (B, 2 * N, C))
    y, s = O.conv_stem_fwd(x, p)
    assert y.shape == (B * N, h)
    R = synth.normal(9326, y.shape)
    dx, g = O.conv_stem_bwd(R, p, s)
    loss = lambda pp, xx=x: float((O.conv_stem_fwd(xx, pp)[0] * R).sum())
    for key in p:
        D = synth.normal(9330 + len(key), p[key].shape)
        pp, pm = dict(p), dict(p)
        pp[key] = p[key] + 1e-6 * D; pm[key] = p[key] - 1e-6 * D
        assert (loss(pp) - loss(pm)) / 2e-6 == pytest.approx(float((g[key] * D).sum()), rel=1e-6, abs=1e-8), key
    D = synth.normal(9340, x.shape)
    assert (loss(p, x + 1e-6 * D) - loss(p, x - 1e-6 * D)) / 2e-6 == pytest.approx(float((dx * D).sum()), rel=1e-6, abs=1e-8)


# --------------------------------------------------------------------------- AdamW
def test_adamw_first_step_closed_form():
    # zero moments, step 1: mhat = g, vhat = g^2, so p' = p - lr (g/(|g|+eps) + wd p)
    p = synth.normal(9100, (50,)); g = synth.normal(9101, (50,))
    lr, b1, b2, eps, wd = 1e-2, 0.9, 0.999, 1e-8, 0.1
    p1, m1, v1 = O.adamw_step(p, g, np.zeros(50), np.zeros(50), 1, lr, b1, b2, eps, wd)
    assert np.allclose(p1, p - lr * (g / (np.abs(g) + eps) + wd * p), rtol=0, atol=1e-15)
    assert np.allclose(m1, 0.1 * g, atol=1e-16) and np.allclose(v1, 0.001 * g * g, atol=1e-18)


def test_adamw_zero_gradient_is_pure_decay():
    p = synth.normal(9102, (20,))
    q, m, v = p.copy(), np.zeros(20), np.zeros(20)
    for t in range(1, 6):
        q, m, v = O.adamw_step(q, np.zeros(20), m, v, t, 0.05, 0.9, 0.999, 1e-8, 0.2)
    assert np.allclose(q, p * (1.0 - 0.05 * 0.2) ** 5, rtol=1e-14)


def test_adamw_matches_library_over_several_steps():
    p0 = synth.normal(9103, (33,))
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.AdamW([tp], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.05)
    p, m, v = p0.copy(), np.zeros(33), np.zeros(33)
    for t in range(1, 8):
        g = synth.normal(9110 + t, (33,))
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        p, m, v = O.adamw_step(p, g, m, v, t, 3e-3, 0.9, 0.95, 1e-8, 0.05)
    # the library writes the same update as p (1 - lr wd) - lr mhat / (sqrt vhat + eps)
    assert np.allclose(p, tp.detach().numpy(), rtol=0, atol=1e-13)
    assert np.abs(p - p0).max() > 1e-3
