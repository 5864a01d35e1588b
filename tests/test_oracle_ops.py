"""Pins for the CPU checker's elementary operations: brute force, closed forms,
invariants and scalar library references.  None of these re-type the checker's own
formula; each would fail on a dropped term, a wrong sign or a transposed operand."""
import math

import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth


def fd(fun, x, dx, step=1e-5):
    return (fun(x + step * dx) - fun(x - step * dx)) / (2 * step)


# ---------------------------------------------------------------------------- linear
def test_linear_matches_triple_loop():
    x = synth.normal(1, (5, 7)); W = synth.normal(2, (7, 3)); b = synth.normal(3, (3,))
    y = O.linear_fwd(x, W, b)
    for i in range(5):
        for j in range(3):
            acc = 0.0
            for k in range(7):
                acc += x[i, k] * W[k, j]
            assert abs(y[i, j] - (acc + b[j])) < 1e-12


def test_linear_identity_weight():
    x = synth.normal(4, (6, 6)); b = synth.normal(5, (6,))
    assert np.allclose(O.linear_fwd(x, np.eye(6), b), x + b, atol=0)


def test_linear_bwd_triple_loop_and_fd():
    x = synth.normal(6, (4, 5)); W = synth.normal(7, (5, 3)); dy = synth.normal(8, (4, 3))
    dx, dW, db = O.linear_bwd(x, W, dy)
    for i in range(4):
        for k in range(5):
            assert abs(dx[i, k] - sum(dy[i, j] * W[k, j] for j in range(3))) < 1e-12
    for k in range(5):
        for j in range(3):
            assert abs(dW[k, j] - sum(x[i, k] * dy[i, j] for i in range(4))) < 1e-12
    for j in range(3):
        assert abs(db[j] - sum(dy[i, j] for i in range(4))) < 1e-12
    R = synth.normal(9, (5, 3))
    num = fd(lambda W_: (O.linear_fwd(x, W_) * dy).sum(), W, R)
    assert abs(num - (dW * R).sum()) < 1e-8


# ------------------------------------------------------------------------- LayerNorm
def test_layernorm_zero_mean_unit_variance():
    x = synth.normal(10, (9, 64), 3.0, 5.0)
    y = O.layernorm_fwd(x, np.ones(64), np.zeros(64), 1e-5)
    assert np.abs(y.mean(axis=1)).max() < 1e-6
    var = x.var(axis=1)
    assert np.allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)


def test_layernorm_affine_and_scale_invariance():
    x = synth.normal(11, (3, 32)); g = synth.normal(12, (32,)); b = synth.normal(13, (32,))
    y0 = O.layernorm_fwd(x, np.ones(32), np.zeros(32), 1e-5)
    assert np.allclose(O.layernorm_fwd(x, g, b, 1e-5), g * y0 + b, atol=1e-14)
    assert np.allclose(O.layernorm_fwd(7.0 * x, g, b, 0.0), O.layernorm_fwd(x, g, b, 0.0), atol=1e-12)


def test_layernorm_bwd_invariants_and_fd():
    x = synth.normal(14, (5, 24)); g = 1 + synth.normal(15, (24,), 0, 0.3)
    b = synth.normal(16, (24,)); dy = synth.normal(17, (5, 24))
    eps = 1e-5
    dx, dg, db = O.layernorm_bwd(x, g, dy, eps)
    mu = x.mean(1, keepdims=True); xhat = (x - mu) / np.sqrt(x.var(1, keepdims=True) + eps)
    assert np.abs(dx.sum(1)).max() < 1e-12
    # the projection onto xhat vanishes exactly only as eps -> 0
    dx0, _, _ = O.layernorm_bwd(x, g, dy, 0.0)
    xhat0 = (x - mu) / np.sqrt(x.var(1, keepdims=True))
    assert np.abs((dx0 * xhat0).sum(1)).max() < 1e-12
    v = x.var(1)
    assert np.allclose((dx * xhat).sum(1), (dy * g * xhat).sum(1) * eps / (v + eps) ** 1.5, rtol=1e-8)
    f = lambda x_: (O.layernorm_fwd(x_, g, b, eps) * dy).sum()
    R = synth.normal(18, x.shape)
    assert abs(fd(f, x, R) - (dx * R).sum()) < 1e-7
    Rg = synth.normal(19, g.shape)
    assert abs(fd(lambda g_: (O.layernorm_fwd(x, g_, b, eps) * dy).sum(), g, Rg) - (dg * Rg).sum()) < 1e-7
    assert np.allclose(db, dy.sum(0))


# --------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_mean_square():
    x = synth.normal(20, (7, 48), 1.0, 2.0)
    y = O.rmsnorm_fwd(x, np.ones(48), 1e-5)
    m = (x * x).mean(1)
    assert np.allclose((y * y).mean(1), m / (m + 1e-5), rtol=1e-12)


def test_rmsnorm_bwd_closed_form_and_fd():
    x = synth.normal(21, (4, 20)); g = 1 + synth.normal(22, (20,), 0, 0.3); dy = synth.normal(23, (4, 20))
    eps = 1e-3
    dx, dg = O.rmsnorm_bwd(x, g, dy, eps)
    r = 1 / np.sqrt((x * x).mean(1) + eps)
    t = dy * g
    # sum_j dx_j x_j = eps * r^3 * sum_j t_j x_j
    assert np.allclose((dx * x).sum(1), eps * r ** 3 * (t * x).sum(1), rtol=1e-10)
    R = synth.normal(24, x.shape)
    assert abs(fd(lambda x_: (O.rmsnorm_fwd(x_, g, eps) * dy).sum(), x, R) - (dx * R).sum()) < 1e-7
    Rg = synth.normal(25, g.shape)
    assert abs(fd(lambda g_: (O.rmsnorm_fwd(x, g_, eps) * dy).sum(), g, Rg) - (dg * Rg).sum()) < 1e-7


# ----------------------------------------------------------------------- activations
def test_gelu_scalar_reference_and_identities():
    z = np.linspace(-6, 6, 97)
    ref = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in z])
    assert np.allclose(O.gelu(z), ref, atol=1e-15)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_grad(np.array([0.0]))[0] - 0.5) < 1e-15
    assert abs(O.gelu(np.array([12.0]))[0] - 12.0) < 1e-12
    assert np.allclose(O.gelu(-z), O.gelu(z) - z, atol=1e-14)
    num = (O.gelu(z + 1e-6) - O.gelu(z - 1e-6)) / 2e-6
    assert np.allclose(O.gelu_grad(z), num, atol=1e-8)


def test_silu_and_swiglu():
    z = np.linspace(-8, 8, 65)
    ref = np.array([t / (1 + math.exp(-t)) for t in z])
    assert np.allclose(O.silu(z), ref, atol=1e-15)
    assert O.silu(np.array([0.0]))[0] == 0.0
    assert abs(O.silu_grad(np.array([0.0]))[0] - 0.5) < 1e-15
    num = (O.silu(z + 1e-6) - O.silu(z - 1e-6)) / 2e-6
    assert np.allclose(O.silu_grad(z), num, atol=1e-8)
    gate = synth.normal(30, (3, 5)); up = synth.normal(31, (3, 5)); da = synth.normal(32, (3, 5))
    dg, du = O.swiglu_bwd(gate, up, da)
    Rg = synth.normal(33, gate.shape); Ru = synth.normal(34, up.shape)
    assert abs(fd(lambda g_: (O.swiglu_fwd(g_, up) * da).sum(), gate, Rg) - (dg * Rg).sum()) < 1e-8
    assert abs(fd(lambda u_: (O.swiglu_fwd(gate, u_) * da).sum(), up, Ru) - (du * Ru).sum()) < 1e-8


# ------------------------------------------------------------------------- attention
def naive_attention(q, k, v, causal):
    """Independent per-row python-loop softmax attention."""
    N, d = q.shape
    o = np.zeros_like(q)
    for i in range(N):
        jmax = i + 1 if causal else N
        s = [sum(q[i, c] * k[j, c] for c in range(d)) / math.sqrt(d) for j in range(jmax)]
        m = max(s)
        e = [math.exp(t - m) for t in s]
        z = sum(e)
        for c in range(d):
            o[i, c] = sum(e[j] / z * v[j, c] for j in range(jmax))
    return o


@pytest.mark.parametrize("causal", [0, 1])
def test_attention_matches_naive_loops(causal):
    q = synth.normal(40, (6, 4)); k = synth.normal(41, (6, 4)); v = synth.normal(42, (6, 4))
    o, P = O.attention_head_fwd(q, k, v, causal)
    assert np.allclose(o, naive_attention(q, k, v, causal), atol=1e-13)
    assert np.abs(P.sum(1) - 1).max() < 1e-12
    if causal:
        assert (np.triu(P, 1) == 0).all()


def test_attention_special_cases():
    v = synth.normal(43, (5, 3)); q = synth.normal(44, (5, 3))
    k = np.tile(synth.normal(45, (1, 3)), (5, 1))
    o, _ = O.attention_head_fwd(q, k, v, 0)
    assert np.allclose(o, np.tile(v.mean(0), (5, 1)), atol=1e-13)
    o, _ = O.attention_head_fwd(q, k, v, 1)
    pref = np.cumsum(v, 0) / np.arange(1, 6)[:, None]
    assert np.allclose(o, pref, atol=1e-13)
    o, _ = O.attention_head_fwd(q[:1], k[:1], v[:1], 1)
    assert np.array_equal(o, v[:1])


def test_attention_causal_future_independence_and_permutation():
    q = synth.normal(46, (7, 4)); k = synth.normal(47, (7, 4)); v = synth.normal(48, (7, 4))
    o1, _ = O.attention_head_fwd(q, k, v, 1)
    k2, v2 = k.copy(), v.copy(); k2[5:] += 3.0; v2[5:] -= 2.0
    o2, _ = O.attention_head_fwd(q, k2, v2, 1)
    assert np.array_equal(o1[:5], o2[:5])
    perm = np.array([3, 0, 6, 2, 5, 1, 4])
    o3, _ = O.attention_head_fwd(q[perm], k[perm], v[perm], 0)
    o0, _ = O.attention_head_fwd(q, k, v, 0)
    assert np.allclose(o3, o0[perm], atol=1e-13)


@pytest.mark.parametrize("causal", [0, 1])
def test_attention_bwd_fd_and_ds_rows(causal):
    q = synth.normal(50, (6, 4)); k = synth.normal(51, (6, 4)); v = synth.normal(52, (6, 4))
    do = synth.normal(53, (6, 4))
    _, P = O.attention_head_fwd(q, k, v, causal)
    dq, dk, dv = O.attention_head_bwd(q, k, v, P, do)
    f = lambda q_, k_, v_: (O.attention_head_fwd(q_, k_, v_, causal)[0] * do).sum()
    R = synth.normal(54, (6, 4))
    assert abs(fd(lambda t: f(t, k, v), q, R) - (dq * R).sum()) < 1e-8
    assert abs(fd(lambda t: f(q, t, v), k, R) - (dk * R).sum()) < 1e-8
    assert abs(fd(lambda t: f(q, k, t), v, R) - (dv * R).sum()) < 1e-8
    dP = do @ v.T
    dS = P * (dP - (P * dP).sum(1, keepdims=True))
    assert np.abs(dS.sum(1)).max() < 1e-13
    # D_i can equally be computed from the output
    o, _ = O.attention_head_fwd(q, k, v, causal)
    assert np.allclose((P * dP).sum(1), (do * o).sum(1), atol=1e-13)


def test_packed_attention_layout_and_lse():
    B, N, H, d = 2, 5, 3, 4
    h = H * d
    qkv = synth.normal(55, (B * N, 3 * h))
    o = O.attention_fwd(qkv, B, N, H, 1)
    b, t = 1, 2
    rows = slice(b * N, (b + 1) * N)
    q = qkv[rows, t * d:(t + 1) * d]; k = qkv[rows, h + t * d:h + (t + 1) * d]
    v = qkv[rows, 2 * h + t * d:2 * h + (t + 1) * d]
    assert np.allclose(o[rows, t * d:(t + 1) * d], naive_attention(q, k, v, 1), atol=1e-13)
    lse = O.attention_lse(qkv, B, N, H, 1)
    for i in range(N):
        s = [(q[i] * k[j]).sum() / math.sqrt(d) for j in range(i + 1)]
        assert abs(lse[b, t, i] - math.log(sum(math.exp(x) for x in s))) < 1e-12
    do = synth.normal(56, (B * N, h))
    dqkv = O.attention_bwd(qkv, do, B, N, H, 1)
    R = synth.normal(57, qkv.shape)
    num = fd(lambda z: (O.attention_fwd(z, B, N, H, 1) * do).sum(), qkv, R)
    assert abs(num - (dqkv * R).sum()) < 1e-7


# ------------------------------------------------------------------------------- MSE
def test_mse():
    y = synth.normal(60, (4, 6)); t = synth.normal(61, (4, 6))
    assert O.mse_fwd(y, y) == 0.0 and not O.mse_bwd(y, y).any()
    assert O.mse_fwd(y, t) >= 0
    assert abs(O.mse_fwd(y, t) - sum((y[i, j] - t[i, j]) ** 2 for i in range(4) for j in range(6)) / 24) < 1e-14
    R = synth.normal(62, y.shape)
    assert abs(fd(lambda y_: O.mse_fwd(y_, t), y, R) - (O.mse_bwd(y, t) * R).sum()) < 1e-9


# ---------------------------------------------------------------------- stems, chain
def test_unfold_order():
    img = np.arange(2 * 3 * 4 * 6, dtype=np.float64).reshape(2, 3, 4, 6)
    out = O.unfold_patches(img, 2)
    assert out.shape == (2 * 2 * 3, 12)
    b, py, px, c, i, j = 1, 1, 2, 2, 1, 0
    assert out[(b * 2 + py) * 3 + px, (c * 2 + i) * 2 + j] == img[b, c, py * 2 + i, px * 2 + j]


def test_embedding_repeated_ids():
    ids = np.array([[1, 3, 1], [1, 0, 3]], dtype=np.int32)
    table = synth.normal(63, (4, 5))
    assert np.array_equal(O.embedding_fwd(ids, table)[2], table[1])
    dy = synth.normal(64, (6, 5))
    dt = O.embedding_bwd(ids, dy, 4)
    assert np.allclose(dt[1], dy[0] + dy[2] + dy[3]) and np.allclose(dt[3], dy[1] + dy[5])
    assert not dt[2].any()


def test_concat_split_roundtrip():
    a = synth.normal(65, (2 * 3, 4)); b = synth.normal(66, (2 * 5, 4))
    c = O.concat_tokens(a, b, 2, 3, 5)
    assert np.array_equal(c[8:11], a[3:6]) and np.array_equal(c[11:16], b[5:10])
    a2, b2 = O.split_tokens(c, 2, 3, 5)
    assert np.array_equal(a, a2) and np.array_equal(b, b2)


def test_concat_split_with_per_sample_image_token_counts():
    """Written-out case: 2 samples, 3 image tokens each, sequence 5, counts (1, 3)."""
    n_img, N, h = 3, 5, 2
    img = np.arange(2 * n_img * h, dtype=np.float64).reshape(2 * n_img, h) + 100.0
    txt = np.arange(2 * N * h, dtype=np.float64).reshape(2 * N, h) + 500.0       # one row per sequence position
    c = O.concat_tokens_counts(img, txt, 2, n_img, N, [1, 3])
    want = np.stack([img[0], txt[1], txt[2], txt[3], txt[4],            # sample 0: one image token, four text rows
                     img[3], img[4], img[5], txt[8], txt[9]])           # sample 1: three image tokens, two text rows
    assert np.array_equal(c, want)
    # with every count at n_img it is the plain concatenation of the image tokens and the last N - n_img positions
    full = O.concat_tokens_counts(img, txt, 2, n_img, N, [3, 3])
    plain = O.concat_tokens(img, np.concatenate([txt[3:5], txt[8:10]]), 2, n_img, N - n_img)
    assert np.array_equal(full, plain)
    # the split is the transpose: <concat(a, b), d> == <a, di> + <b, dt> for any d
    d = synth.normal(67, (2 * N, h))
    di, dt = O.split_tokens_counts(d, 2, n_img, N, [1, 3])
    assert abs((c * d).sum() - ((img * di).sum() + (txt * dt).sum())) < 1e-9
    assert not di[1:3].any() and not dt[0].any() and not dt[5:8].any()     # unused image tokens, image positions
    assert np.array_equal(di[0], d[0]) and np.array_equal(dt[1:5], d[1:5]) and np.array_equal(di[3:6], d[5:8])


# ------------------------------------------------------------------- stage semantics
def test_stage_time_semantics():
    assert O.time_sliced([3.0, 4.5]) == 7.5      # Eq. 1
    assert O.colocated([3.0, 4.5]) == 4.5        # Eq. 4
    curves = [{64: 10.0, 128: 6.0, 192: 5.0}, {64: 30.0, 128: 16.0, 192: 11.0}]
    q, t = O.best_split(curves, 256)
    assert q == [64, 192] and t == 11.0          # Eq. 4 under Eq. 5
    q, t = O.best_split(curves, 192)
    assert q == [64, 128] and t == 16.0
    assert abs(O.interference_delta((0.1, 2.0, 3.0), [0.5, 0.25]) - (0.1 + 1.5 + 0.375)) < 1e-15


def test_synth_determinism_and_moments():
    a = synth.normal(70, (100000,)); b = synth.normal(70, (100000,))
    assert np.array_equal(a, b)
    assert abs(a.mean()) < 0.02 and abs(a.std() - 1) < 0.02
    u = synth.uniform(71, (100000,))
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 0.01
    i = synth.integers(72, (1000,), 0, 1000)
    assert i.min() >= 0 and i.max() < 1000
    # prefix property of the counter-based generator
    assert np.array_equal(synth.normal(70, (10,)), a[:10])
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415926], dtype=np.float32)
    r = synth.round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625
    assert np.array_equal(synth.from_bf16_bits(synth.to_bf16_bits(x)), r)
