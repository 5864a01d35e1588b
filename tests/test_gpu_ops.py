"""Kernel-level parity: each operation called through the C ABI against the CPU checker
on the same seeded inputs, at sizes that span several tiles and a ragged tail, plus
bit-identity of the outputs across CU quotas."""
import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import rel_l2, quantize, to_dev, from_dev, tol, assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
QUOTAS = [256, 64, 24]


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_18710_amd import binding
    binding.lib()
    return binding


def empty(shape, dtype):
    return torch.empty(shape, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy().copy()


LINEAR_SHAPES = [
    ("f32", 77, 40, 52), ("f32", 256, 128, 384),
    ("bf16", 333, 264, 392),          # ragged in every dimension, several 128-tiles
    ("bf16", 1568, 768, 2304),        # ViT QKV projection of the CLIP-B-scale workload
    ("bf16", 4096, 512, 8192),        # enough tiles for the 256x256 configuration
    ("bf16", 40, 24, 16), ("bf16", 129, 600, 136),
    ("bf16", 4104, 520, 264),         # long contraction over few output tiles: split weight gradient
    ("bf16", 2100, 520, 1304),        # at 24 CUs: whole rounds of large tiles + a quarter-tile tail with ragged edges
]


@pytest.mark.parametrize("dtype,T,k,n", LINEAR_SHAPES)
def test_linear_fwd_dgrad_wgrad(mb, dtype, T, k, n):
    X = quantize(synth.normal(1, (T, k)), dtype); W = quantize(synth.normal(2, (k, n), 0, 0.05), dtype)
    b = quantize(synth.normal(3, (n,), 0, 0.1), dtype); R = quantize(synth.normal(4, (T, n)), dtype)
    dY = quantize(synth.normal(5, (T, n)), dtype); Rk = quantize(synth.normal(6, (T, k)), dtype)
    dX_, W_, b_, R_, dY_, Rk_ = [to_dev(a, dtype) for a in (X, W, b, R, dY, Rk)]
    ref_y = O.linear_fwd(X, W, b) + R
    ref_dx, ref_dw, ref_db = O.linear_bwd(X, W, dY)
    ref_dx = ref_dx + Rk
    outs = []
    for q in QUOTAS:
        Y = empty((T, n), dtype); dX = empty((T, k), dtype); dW = empty((k, n), dtype); db = empty((n,), dtype)
        scratch = torch.empty(mb.linear_wgrad_scratch_bytes(T, k, n), dtype=torch.uint8, device="cuda")
        mb.op_linear_fwd(None, q, dtype, T, k, n, dX_, W_, b_, R_, Y)
        mb.op_linear_dgrad(None, q, dtype, T, k, n, dY_, W_, Rk_, dX)
        mb.op_linear_wgrad(None, q, dtype, T, k, n, dX_, dY_, dW, db, scratch)
        torch.cuda.synchronize()
        outs.append([bits(t) for t in (Y, dX, dW, db)])
        if q == QUOTAS[0]:
            # the stated relative L2 tolerance and, element by element, one rounding of an fp32 sum
            assert_close(from_dev(Y), ref_y, dtype, "Y")
            assert_close(from_dev(dX), ref_dx, dtype, "dX")
            assert_close(from_dev(dW), ref_dw, dtype, "dW")
            assert_close(from_dev(db), ref_db, dtype, "db")
    for o in outs[1:]:
        for a, b0 in zip(o, outs[0]):
            assert np.array_equal(a, b0), "result depends on the quota"


@pytest.mark.parametrize("T,k,n", [(2100, 1304, 520), (4096, 2048, 1536), (1000, 520, 4104)])
def test_linear_dgrad_without_residual_partial_round(mb, T, k, n):
    """Input gradient with nothing added in the epilogue (the plain store path), at quotas that
    leave a partial round of large tiles to the quarter-tile launch (ragged edges in the first
    shape, a long contraction over few tiles in the last); bits must not depend on the quota."""
    W = quantize(synth.normal(21, (k, n), 0, 0.05), "bf16"); dY = quantize(synth.normal(22, (T, n)), "bf16")
    W_, dY_ = to_dev(W, "bf16"), to_dev(dY, "bf16")
    ref_dx, _, _ = O.linear_bwd(np.zeros((T, k)), W, dY)
    outs = []
    for q in (256, 24, 40, 8):
        dX = empty((T, k), "bf16")
        mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, None, dX)
        torch.cuda.synchronize()
        outs.append(bits(dX))
        if q == 256:
            assert_close(from_dev(dX), ref_dx, "bf16", "dX")
    for o in outs[1:]:
        assert np.array_equal(o, outs[0]), "result depends on the quota"


@pytest.mark.parametrize("T,k,n,with_res", [(1000, 504, 384, False), (1000, 504, 384, True), (2048, 1024, 2304, True),
                                             (777, 264, 128, False)])
def test_linear_dgrad_four_wave_kernel_matches_the_other_kernels_bit_for_bit(mb, T, k, n, with_res):
    """Contractions that are a multiple of 128 long send whole 256x256 tiles of the input
    gradient to the four-wave kernel; the quotas below make the host pick it for all tiles (8),
    for the whole rounds only (the rest goes to the quarter-tile kernel), or not at all (plans
    of 128x128 tiles).  Ragged edges in both output dimensions, with and without the residual
    added in the epilogue; every element against the oracle, and the bits must not depend on
    which kernel produced them."""
    W = quantize(synth.normal(31, (k, n), 0, 0.05), "bf16"); dY = quantize(synth.normal(32, (T, n)), "bf16")
    R = quantize(synth.normal(33, (T, k)), "bf16") if with_res else None
    W_, dY_ = to_dev(W, "bf16"), to_dev(dY, "bf16")
    R_ = to_dev(R, "bf16") if with_res else None
    ref_dx, _, _ = O.linear_bwd(np.zeros((T, k)), W, dY)
    if with_res:
        ref_dx = ref_dx + R
    outs = []
    for q in (8, 16, 3, 256, 40):
        dX = empty((T, k), "bf16")
        mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, R_, dX)
        torch.cuda.synchronize()
        outs.append(bits(dX))
        if q == 8:
            got = from_dev(dX)
            assert rel_l2(got, ref_dx) <= 2e-2
            # element by element: one bf16 rounding of an fp32 sum of n products
            tol = 2.0 ** -7 * np.abs(ref_dx) + 1e-2 * np.sqrt(n) * 0.05
            assert np.all(np.abs(got - ref_dx) <= tol)
    for o in outs[1:]:
        assert np.array_equal(o, outs[0]), "result depends on the quota"


def test_linear_without_bias_and_residual_and_empty(mb):
    T, k, n = 70, 64, 72
    X = quantize(synth.normal(7, (T, k)), "bf16"); W = quantize(synth.normal(8, (k, n), 0, 0.05), "bf16")
    Y = empty((T, n), "bf16")
    mb.op_linear_fwd(None, 256, "bf16", T, k, n, to_dev(X, "bf16"), to_dev(W, "bf16"), None, None, Y)
    torch.cuda.synchronize()
    assert rel_l2(from_dev(Y), X @ W) <= 2e-2
    mb.op_linear_fwd(None, 256, "bf16", 0, k, n, to_dev(X, "bf16"), to_dev(W, "bf16"), None, None, Y)   # no tokens: no-op
    with pytest.raises(mb.MosaicError) as e:
        mb.op_linear_fwd(None, 0, "bf16", T, k, n, Y, Y, None, None, Y)
    assert e.value.status == mb.EQUOTA
    with pytest.raises(mb.MosaicError) as e:
        mb.op_linear_fwd(None, 64, "bf16", T, k, n, None, Y, None, None, Y)
    assert e.value.status == mb.EINVAL


ATTN_SHAPES = [("f32", 2, 16, 4, 32, 0), ("f32", 2, 128, 4, 32, 1), ("f32", 1, 37, 2, 24, 1),
               ("bf16", 2, 196, 3, 64, 0), ("bf16", 1, 300, 2, 128, 1), ("bf16", 2, 1, 2, 64, 1),
               ("bf16", 1, 1024, 2, 128, 1), ("bf16", 2, 577, 2, 64, 0), ("bf16", 1, 129, 1, 64, 1),
               ("bf16", 1, 200, 2, 32, 1),
               # many heads over few workgroups: several rounds of the head-by-head work order,
               # mirrored on odd rounds (3 tiles per head), and a head count that is not a
               # multiple of the XCD count
               ("bf16", 2, 384, 19, 64, 1), ("bf16", 3, 100, 20, 64, 0)]


@pytest.mark.parametrize("dtype,B,N,H,d,causal", ATTN_SHAPES)
def test_attention_fwd_bwd(mb, dtype, B, N, H, d, causal):
    h = H * d
    qkv = quantize(synth.normal(10, (B * N, 3 * h)), dtype)
    dO = quantize(synth.normal(11, (B * N, h)), dtype)
    ref_o = O.attention_fwd(qkv, B, N, H, causal)
    ref_lse = O.attention_lse(qkv, B, N, H, causal)
    ref_d = O.attention_bwd(qkv, dO, B, N, H, causal)
    qkv_, dO_ = to_dev(qkv, dtype), to_dev(dO, dtype)
    outs = []
    for q in QUOTAS:
        Oo = empty((B * N, h), dtype); lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        dqkv = empty((B * N, 3 * h), dtype); delta = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        mb.op_attention_fwd(None, q, dtype, B, N, H, d, causal, qkv_, Oo, lse)
        mb.op_attention_bwd(None, q, dtype, B, N, H, d, causal, qkv_, Oo, lse, dO_, dqkv, delta)
        torch.cuda.synchronize()
        outs.append([bits(Oo), bits(lse), bits(dqkv)])
        if q == QUOTAS[0]:
            # element by element too: the probabilities and dS are rounded to bf16 before their products, and
            # dS = P (dP - delta) cancels where a row's probability sits on few keys, so the rounding of O
            # inside delta shows: the gradients get a wider floor than a chain of plain roundings would
            assert_close(from_dev(Oo), ref_o, dtype, "O", roundings=2)
            assert_close(from_dev(lse), ref_lse, dtype, "lse", l2=(1e-5 if dtype == "f32" else 1e-2))
            got = from_dev(dqkv)
            for part in range(3):      # dq, dk, dv separately
                assert_close(got[:, part * h:(part + 1) * h], ref_d[:, part * h:(part + 1) * h], dtype, ("dq", "dk", "dv")[part], roundings=8)
    for o in outs[1:]:
        for a, b0 in zip(o, outs[0]):
            assert np.array_equal(a, b0)


@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("kind", ["rising", "steep", "falling", "spike"])
def test_attention_forward_when_the_row_maximum_moves_late(mb, kind, causal):
    """The forward kernel at head size 128 forms a block's probabilities against the reference
    its row already has and repairs the block when they come out too large.  Scores that keep
    rising along the keys by more than sixteen powers of two per block of 32 send every block
    through that repair; falling scores and a single late spike take the other roads."""
    B, N, H, d = 2, 416, 2, 128          # 13 key blocks, ragged last query tile
    h = H * d
    rng = np.random.default_rng(77)
    q = np.ones((B * N, h)) + 0.05 * rng.standard_normal((B * N, h))
    j = np.tile(np.arange(N), B)[:, None].astype(np.float64)
    if kind == "rising":
        k = (0.06 * j) * np.ones((1, h))                  # score rises by 0.06 * 128 / sqrt(128) * 32 = 21.7 nats per block
    elif kind == "steep":
        k = (0.3 * j) * np.ones((1, h))                   # 156 powers of two per block: the first attempt overflows to infinity
    elif kind == "falling":
        k = (0.06 * (N - j)) * np.ones((1, h))
    else:
        k = 0.02 * rng.standard_normal((B * N, h))
        k[(np.arange(B * N) % N) == 300] = 1.5           # one key far above the rest, in the tenth block
    k = k + 0.02 * rng.standard_normal((B * N, h))
    v = rng.standard_normal((B * N, h))
    qkv = quantize(np.concatenate([q, k, v], 1), "bf16")
    ref_o = O.attention_fwd(qkv, B, N, H, causal)
    ref_lse = O.attention_lse(qkv, B, N, H, causal)
    qkv_ = to_dev(qkv, "bf16")
    outs = []
    for quota in (256, 24):
        Oo = empty((B * N, h), "bf16"); lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        mb.op_attention_fwd(None, quota, "bf16", B, N, H, d, causal, qkv_, Oo, lse)
        torch.cuda.synchronize()
        outs.append([bits(Oo), bits(lse)])
    assert np.isfinite(from_dev(Oo)).all() and np.isfinite(from_dev(lse)).all()
    assert_close(from_dev(Oo), ref_o, "bf16", "O", roundings=2)
    assert np.abs(from_dev(lse) - ref_lse).max() <= 1e-3 * max(1.0, np.abs(ref_lse).max())
    for a, b0 in zip(outs[1], outs[0]):
        assert np.array_equal(a, b0)


NORM_SHAPES = [("f32", "layernorm", 32, 128), ("f32", "rmsnorm", 256, 128), ("bf16", "layernorm", 1568, 768),
               ("bf16", "rmsnorm", 1000, 2048), ("bf16", "rmsnorm", 130, 5120), ("bf16", "layernorm", 3, 3200),
               ("f32", "layernorm", 5, 24)]


@pytest.mark.parametrize("dtype,norm,T,h", NORM_SHAPES)
def test_norm_fwd_bwd(mb, dtype, norm, T, h):
    eps = 1e-5
    x = quantize(synth.normal(20, (T, h), 0.3, 1.7), dtype)
    g = quantize(1 + synth.normal(21, (h,), 0, 0.1), dtype); b = quantize(synth.normal(22, (h,), 0, 0.1), dtype)
    dy = quantize(synth.normal(23, (T, h)), dtype); R = quantize(synth.normal(24, (T, h)), dtype)
    if norm == "layernorm":
        ref_y = O.layernorm_fwd(x, g, b, eps)
        ref_dx, ref_dg, ref_db = O.layernorm_bwd(x, g, dy, eps)
    else:
        ref_y = O.rmsnorm_fwd(x, g, eps)
        ref_dx, ref_dg = O.rmsnorm_bwd(x, g, dy, eps)
        ref_db = None
    ref_dx = ref_dx + R
    x_, g_, b_, dy_, R_ = [to_dev(a, dtype) for a in (x, g, b, dy, R)]
    outs = []
    for q in QUOTAS:
        y = empty((T, h), dtype); stats = torch.empty((T, 2), dtype=torch.float32, device="cuda")
        dx = empty((T, h), dtype); dg = empty((h,), dtype); db = empty((h,), dtype)
        scratch = torch.empty(mb.norm_bwd_scratch_bytes(h), dtype=torch.uint8, device="cuda")
        mb.op_norm_fwd(None, q, dtype, norm, T, h, eps, x_, g_, b_, y, stats)
        mb.op_norm_bwd(None, q, dtype, norm, T, h, x_, g_, stats, dy_, R_, dx, dg, db, scratch)
        torch.cuda.synchronize()
        outs.append([bits(y), bits(dx), bits(dg)] + ([bits(db)] if ref_db is not None else []))
        if q == QUOTAS[0]:
            assert_close(from_dev(y), ref_y, dtype, "y")
            assert_close(from_dev(dx), ref_dx, dtype, "dx", roundings=2)
            assert_close(from_dev(dg), ref_dg, dtype, "dgamma", roundings=2)
            if ref_db is not None:
                assert_close(from_dev(db), ref_db, dtype, "dbeta")
    for o in outs[1:]:
        for a, b0 in zip(o, outs[0]):
            assert np.array_equal(a, b0)


@pytest.mark.parametrize("dtype,T,f", [("f32", 32, 512), ("bf16", 1568, 3072), ("bf16", 77, 88), ("f32", 256, 384)])
def test_activations(mb, dtype, T, f):
    z = quantize(synth.normal(30, (T, f), 0, 2.0), dtype); da = quantize(synth.normal(31, (T, f)), dtype)
    gu = quantize(synth.normal(32, (T, 2 * f), 0, 2.0), dtype)
    z_, da_, gu_ = to_dev(z, dtype), to_dev(da, dtype), to_dev(gu, dtype)
    outs = []
    for q in QUOTAS:
        a = empty((T, f), dtype); dz = empty((T, f), dtype); s = empty((T, f), dtype); dgu = empty((T, 2 * f), dtype)
        mb.op_gelu_fwd(None, q, dtype, T * f, z_, a)
        mb.op_gelu_bwd(None, q, dtype, T * f, z_, da_, dz)
        mb.op_swiglu_fwd(None, q, dtype, T, f, gu_, s)
        mb.op_swiglu_bwd(None, q, dtype, T, f, gu_, da_, dgu)
        torch.cuda.synchronize()
        outs.append([bits(t) for t in (a, dz, s, dgu)])
        if q == QUOTAS[0]:
            assert_close(from_dev(a), O.gelu(z), dtype, "gelu")
            assert_close(from_dev(dz), da * O.gelu_grad(z), dtype, "gelu grad")
            assert_close(from_dev(s), O.swiglu_fwd(gu[:, :f], gu[:, f:]), dtype, "swiglu")
            dg, du = O.swiglu_bwd(gu[:, :f], gu[:, f:], da)
            assert_close(from_dev(dgu), np.concatenate([dg, du], 1), dtype, "swiglu grad")
    for o in outs[1:]:
        for a0, b0 in zip(o, outs[0]):
            assert np.array_equal(a0, b0)


LINEAR_ACT_SHAPES = [
    # (dtype, act, T, k, n, bias)
    ("bf16", "gelu", 1568, 768, 3072, True),        # ViT MLP up projection: bias + GELU in the epilogue
    ("bf16", "gelu", 333, 264, 392, True),          # ragged in every dimension
    ("bf16", "gelu", 2100, 520, 1304, False),       # at 24 CUs: whole rounds of large tiles + quarter-tile tail
    ("bf16", "gelu_tanh", 300, 128, 256, True),     # no epilogue for this form: the elementwise pass follows
    ("f32", "gelu", 77, 40, 52, True),
    ("bf16", "swiglu", 2100, 520, 2560, False),     # gate | up of 1280 columns each: ten quarter tiles per half
    ("bf16", "swiglu", 512, 256, 11264, False),     # the small decoder's gate/up width
    ("bf16", "swiglu", 700, 264, 1536, True),       # with a bias, ragged rows
    ("bf16", "swiglu", 333, 264, 400, False),       # halves that are not whole tiles wide: product, then the elementwise pass
    ("f32", "swiglu", 64, 40, 104, False),
]


@pytest.mark.parametrize("dtype,act,T,k,n,with_bias", LINEAR_ACT_SHAPES)
def test_linear_with_activation_in_the_epilogue(mb, dtype, act, T, k, n, with_bias):
    """Z = X W + b and A = act(Z) from one call: the bits of the product followed by the separate
    activation pass, for every quota; Z and A against the CPU checker."""
    code = {"gelu": mb.GELU, "swiglu": mb.SWIGLU, "gelu_tanh": mb.GELU_TANH}[act]
    na = n // 2 if act == "swiglu" else n
    X = quantize(synth.normal(61, (T, k)), dtype); W = quantize(synth.normal(62, (k, n), 0, 0.06), dtype)
    b = quantize(synth.normal(63, (n,), 0, 0.3), dtype) if with_bias else None
    X_, W_ = to_dev(X, dtype), to_dev(W, dtype)
    b_ = to_dev(b, dtype) if with_bias else None
    # separate passes
    Z0 = empty((T, n), dtype); A0 = empty((T, na), dtype)
    mb.op_linear_fwd(None, 256, dtype, T, k, n, X_, W_, b_, None, Z0)
    if act == "swiglu":
        mb.op_swiglu_fwd(None, 256, dtype, T, na, Z0, A0)
    elif act == "gelu":
        mb.op_gelu_fwd(None, 256, dtype, T * n, Z0, A0)
    else:
        mb.op_gelu_tanh_fwd(None, 256, dtype, T * n, Z0, A0)
    torch.cuda.synchronize()
    ref_z = O.linear_fwd(X, W, b)
    if act == "swiglu":
        ref_a = O.swiglu_fwd(ref_z[:, :na], ref_z[:, na:])
    elif act == "gelu":
        ref_a = O.gelu(ref_z)
    else:
        ref_a = O.gelu_tanh(ref_z)
    for q in [256, 64, 24, 232]:
        Z = torch.full((T, n), float("nan"), dtype=Z0.dtype, device="cuda")
        A = torch.full((T, na), float("nan"), dtype=Z0.dtype, device="cuda")
        mb.op_linear_act_fwd(None, q, dtype, code, T, k, n, X_, W_, b_, Z, A)
        torch.cuda.synchronize()
        assert np.array_equal(bits(Z), bits(Z0)), f"Z differs from the separate product at quota {q}"
        assert np.array_equal(bits(A), bits(A0)), f"A differs from the separate activation pass at quota {q}"
        if q == 256:
            assert_close(from_dev(Z), ref_z, dtype, "Z")
            # the activation is taken of the stored (rounded) Z: one more rounding on its input
            assert_close(from_dev(A), ref_a, dtype, "A", roundings=4 if act == "swiglu" else 2)


def test_linear_with_activation_rejects_bad_arguments(mb):
    x = empty((8, 8), "bf16")
    with pytest.raises(mb.MosaicError):
        mb.op_linear_act_fwd(None, 256, "bf16", 7, 8, 8, 8, x, x, None, x, x)
    with pytest.raises(mb.MosaicError):
        mb.op_linear_act_fwd(None, 256, "bf16", mb.SWIGLU, 8, 8, 7, x, x, None, x, x)
    mb.op_linear_act_fwd(None, 256, "bf16", mb.GELU, 0, 8, 8, x, x, None, x, x)     # nothing to do


@pytest.mark.parametrize("dtype,n", [("f32", 2 * 128 * 128), ("bf16", 8192 * 2048), ("bf16", 8), ("f32", 4 * 1031)])
def test_mse(mb, dtype, n):
    y = quantize(synth.normal(40, (n,)), dtype); t = quantize(synth.normal(41, (n,)), dtype)
    y_, t_ = to_dev(y, dtype), to_dev(t, dtype)
    outs = []
    for q in QUOTAS:
        dy = empty((n,), dtype); loss = torch.empty(1, dtype=torch.float32, device="cuda")
        scratch = torch.empty(mb.mse_scratch_bytes(), dtype=torch.uint8, device="cuda")
        mb.op_mse(None, q, dtype, n, y_, t_, dy, loss, scratch)
        torch.cuda.synchronize()
        outs.append([bits(dy), bits(loss)])
        if q == QUOTAS[0]:
            assert abs(float(loss.item()) - O.mse_fwd(y, t)) <= 1e-5 * O.mse_fwd(y, t)
            assert rel_l2(from_dev(dy), O.mse_bwd(y, t)) <= tol(dtype)
    for o in outs[1:]:
        for a0, b0 in zip(o, outs[0]):
            assert np.array_equal(a0, b0)
