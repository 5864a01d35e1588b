"""Parity at the benchmark's full sizes (configs[1]: CLIP-B / small-LM scale), in the launch
configuration bench.py times.  The oracle cannot run the whole stage here in seconds, so:
  * every output element of a linear layer is an independent dot product and every
    (sample, head) of attention an independent problem: sampled rows / columns / heads are
    checked against the oracle one by one;
  * properties that hold at any size are checked on the full stage: colocated and
    time-sliced execution give identical bits, the loss is finite and positive.
"""
import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import rel_l2, quantize, to_dev, from_dev, assert_close

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_18710_amd import binding
    binding.lib()
    return binding


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy().copy()


def test_decoder_gate_up_projection_sampled(mb):
    """T=8192, k=2048, n=11264: the shape of the roofline entry."""
    T, k, n = 8192, 2048, 11264
    X = quantize(synth.normal(9001, (T, k)), "bf16")
    W = quantize(synth.normal(9002, (k, n), 0, 0.02), "bf16")
    dY = quantize(synth.uniform(9003, (T, n), -1.0, 1.0), "bf16")
    X_, W_, dY_ = to_dev(X, "bf16"), to_dev(W, "bf16"), to_dev(dY, "bf16")
    Y = torch.empty((T, n), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, k), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((k, n), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(mb.linear_wgrad_scratch_bytes(T, k, n), dtype=torch.uint8, device="cuda")
    snaps = []
    for q in (256, 192):
        mb.op_linear_fwd(None, q, "bf16", T, k, n, X_, W_, None, None, Y)
        mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, None, dX)
        mb.op_linear_wgrad(None, q, "bf16", T, k, n, X_, dY_, dW, None, ws)
        torch.cuda.synchronize()
        snaps.append([bits(Y), bits(dX), bits(dW)])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b), "full-size result depends on the quota"
    rows = synth.integers(9004, (48,), 0, T)
    # tile edges, and rows of the tiles that do not fill a whole round of 256 large tiles: the forward
    # form's 1408 tiles leave 128 (the last three of its 32 tile rows, in the last panels) to the
    # quarter-tile launch
    rows[:10] = [0, 255, 256, T - 1, 7424, 7551, 7552, 7679, 7680, 8063]
    Yh, dXh = from_dev(Y[torch.from_numpy(rows).long().cuda()]), from_dev(dX[torch.from_numpy(rows).long().cuda()])
    assert_close(Yh, X[rows] @ W, "bf16", "Y rows")
    assert_close(dXh, dY[rows] @ W.T, "bf16", "dX rows")
    cols = synth.integers(9005, (24,), 0, n)
    # the weight gradient's 352 tiles leave 96 to the quarter-tile launch: the last tile columns
    cols[:8] = [0, 255, n - 1, 8191, 8192, 9215, 10239, 11135]
    dWh = from_dev(dW[:, torch.from_numpy(cols).long().cuda()])
    assert_close(dWh, X.T @ dY[:, cols], "bf16", "dW columns")


@pytest.mark.parametrize("T,k,n,note", [
    (16384, 768, 22016, "258 tiles: 256 in one round, the last two cut into pieces"),
    (16384, 1024, 8448, "132 tiles, more than half a round and less than one, long contraction: all cut into pieces"),
    (12288, 768, 8704, "102 tiles: the whole product cut into 2 pieces"),
    (16384, 1000, 16904, "268 tiles with ragged last tile row and column: the last panel's 12 tiles are the cut ones"),
])
def test_weight_gradient_with_tiles_cut_along_the_contraction(mb, T, k, n, note):
    """Weight gradients whose tile count does not fill rounds of 256: the tiles of the partial round
    are cut along the token dimension, each piece accumulated by its own workgroup, and a second
    pass adds the pieces.  Which tiles are cut depends on the shape alone: same bits at every quota.
    Sampled columns (all rows) against the checker, among them columns of the cut tiles (the end
    of the tile list: the last tile columns) and of uncut ones."""
    X = quantize(synth.normal(9201, (T, k)), "bf16")
    dY = quantize(synth.uniform(9202, (T, n), -1.0, 1.0), "bf16")
    X_, dY_ = to_dev(X, "bf16"), to_dev(dY, "bf16")
    dW = torch.empty((k, n), dtype=torch.bfloat16, device="cuda")
    nbytes = mb.linear_wgrad_scratch_bytes(T, k, n)
    assert nbytes > 4 * 65536 * 2, "this shape is meant to take the split path"
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    snaps = []
    for q in (256, 200, 64):
        dW.fill_(float("nan"))
        mb.op_linear_wgrad(None, q, "bf16", T, k, n, X_, dY_, dW, None, ws)
        torch.cuda.synchronize()
        snaps.append(bits(dW))
    for b in snaps[1:]:
        assert np.array_equal(snaps[0], b), "result depends on the quota"
    cols = synth.integers(9203, (32,), 0, n)
    cols[:10] = [0, 255, 256, n - 1, n - 2, n - 255, n - 256, n - 257, n - 512, n // 2]
    dWh = from_dev(dW[:, torch.from_numpy(cols).long().cuda()])
    assert_close(dWh, X.T @ dY[:, cols], "bf16", "dW columns")


def test_gate_up_projection_with_swiglu_epilogue_at_the_7b_shape_sampled(mb):
    """T=32768, k=4096, n=22016: the dominant product of configs[2] and configs[4], with silu(gate)*up
    written by the epilogue.  Sampled rows of [gate | up] and of the activation against the checker
    (rows at tile edges, and in the tiles of the last, partial round, which the quarter-tile launch
    takes); the activation must equal, bit for bit, the separate pass over the stored product."""
    T, k, f = 32768, 4096, 11008
    n = 2 * f
    X_ = torch.from_numpy(synth.bulk_uniform(9101, (T, k), -1.0, 1.0)).to(torch.bfloat16).cuda()
    W_ = torch.from_numpy(synth.bulk_uniform(9102, (k, n), -0.03, 0.03)).to(torch.bfloat16).cuda()
    Z = torch.empty((T, n), dtype=torch.bfloat16, device="cuda")
    A = torch.empty((T, f), dtype=torch.bfloat16, device="cuda")
    A2 = torch.empty((T, f), dtype=torch.bfloat16, device="cuda")
    snaps = []
    for q in (256, 224):
        Z.fill_(float("nan")); A.fill_(float("nan"))
        mb.op_linear_act_fwd(None, q, "bf16", mb.SWIGLU, T, k, n, X_, W_, None, Z, A)
        torch.cuda.synchronize()
        snaps.append([bits(Z[::97]), bits(A[::97])])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b), "full-size result depends on the quota"
    mb.op_swiglu_fwd(None, 256, "bf16", T, f, Z, A2)
    torch.cuda.synchronize()
    assert torch.equal(A.view(torch.int16), A2.view(torch.int16)), "epilogue activation differs from the separate pass"
    rows = synth.integers(9104, (24,), 0, T)
    rows[:8] = [0, 255, 256, T - 1, T - 256, T - 257, 16383, 16384]
    ridx = torch.from_numpy(rows).long().cuda()
    Xh, Wh = X_[ridx].float().cpu().numpy().astype(np.float64), W_.float().cpu().numpy().astype(np.float64)
    ref_z = Xh @ Wh
    assert_close(from_dev(Z[ridx]), ref_z, "bf16", "[gate | up] rows")
    assert_close(from_dev(A[ridx]), O.swiglu_fwd(ref_z[:, :f], ref_z[:, f:]), "bf16", "activation rows", roundings=4)


def test_decoder_attention_sampled_heads(mb):
    """B=8, N=1024, 16 heads of 128, causal: sampled (sample, head) problems."""
    B, N, H, d = 8, 1024, 16, 128
    h = H * d
    qkv = quantize(synth.normal(9010, (B * N, 3 * h)), "bf16")
    dO = quantize(synth.normal(9011, (B * N, h)), "bf16")
    qkv_, dO_ = to_dev(qkv, "bf16"), to_dev(dO, "bf16")
    Oo = torch.empty((B * N, h), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    dqkv = torch.empty_like(qkv_)
    delta = torch.empty_like(lse)
    snaps = []
    for q in (256, 192):
        mb.op_attention_fwd(None, q, "bf16", B, N, H, d, 1, qkv_, Oo, lse)
        mb.op_attention_bwd(None, q, "bf16", B, N, H, d, 1, qkv_, Oo, lse, dO_, dqkv, delta)
        torch.cuda.synchronize()
        snaps.append([bits(Oo), bits(lse), bits(dqkv)])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b)
    Oh, dh, lh = from_dev(Oo), from_dev(dqkv), from_dev(lse)
    for (b, t) in ((0, 0), (3, 7), (7, 15), (5, 9)):
        rows = slice(b * N, (b + 1) * N)
        c = slice(t * d, (t + 1) * d)
        qh, kh, vh = qkv[rows, 0:h][:, c], qkv[rows, h:2 * h][:, c], qkv[rows, 2 * h:][:, c]
        o_ref, P = O.attention_head_fwd(qh, kh, vh, 1)
        dq, dk, dv = O.attention_head_bwd(qh, kh, vh, P, dO[rows, c])
        assert_close(Oh[rows, c], o_ref, "bf16", ("O", b, t), roundings=2)
        assert_close(dh[rows, t * d:(t + 1) * d], dq, "bf16", ("dq", b, t), roundings=8)
        assert_close(dh[rows, h + t * d:h + (t + 1) * d], dk, "bf16", ("dk", b, t), roundings=8)
        assert_close(dh[rows, 2 * h + t * d:2 * h + (t + 1) * d], dv, "bf16", ("dv", b, t), roundings=8)
        S = (qh @ kh.T) / np.sqrt(d)
        S = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, S)
        mx = S.max(-1)
        assert rel_l2(lh[b, t], mx + np.log(np.exp(S - mx[:, None]).sum(-1))) <= 1e-2


def test_full_stage_modes_are_bit_identical(mb):
    """The benchmarked stage itself: colocated (64/192 CUs) and time-sliced runs of all
    three modules give the same bits in every output, input gradient and parameter
    gradient, and the decoder's loss is finite."""
    from paper_2605_18710_amd.workload import StagedStage
    stage = StagedStage(1)
    cus = mb.device_cu_count()
    mb.pool_reserve(cus, 0, mb.STRIPED)
    stage.reserve([64, 192])
    snaps = []
    for quotas, mode in (([cus], mb.TIME_SLICED), ([64, 192], mb.COLOCATED)):
        for m in stage.staged:
            m.module.grads.zero_()
        r = stage.run(quotas, mode)
        assert r["stage_ms"] > 0
        snaps.append([bits(m.y) for m in stage.staged] + [bits(m.dx) for m in stage.staged] +
                     [bits(m.module.grads) for m in stage.staged] + [bits(stage.staged[-1].loss)])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b), "colocated and time-sliced runs differ at full size"
    loss = float(stage.staged[-1].loss.item())
    assert np.isfinite(loss) and loss > 0
    for m in stage.staged:
        g = m.module.grads.float()
        assert torch.isfinite(g).all() and float(g.abs().max()) > 0
    stage.destroy()


def _linear_three_forms(mb, T, k, n, seed, quotas=(256, 192)):
    """Runs forward / input-gradient / weight-gradient of one linear layer at full shape for
    two quotas, checks the bits agree, and returns host inputs and device outputs.  Activations
    are drawn uniform in [-2, 2) here: the counter-based normal generator needs several
    seconds per 10^7 values on the host and these operands hold 10^8."""
    X = quantize(synth.uniform(seed, (T, k), -2.0, 2.0), "bf16")
    W = quantize(synth.normal(seed + 1, (k, n), 0, 0.02), "bf16")
    dY = quantize(synth.uniform(seed + 2, (T, n), -1.0, 1.0), "bf16")
    X_, W_, dY_ = to_dev(X, "bf16"), to_dev(W, "bf16"), to_dev(dY, "bf16")
    Y = torch.empty((T, n), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, k), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((k, n), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(1, mb.linear_wgrad_scratch_bytes(T, k, n)), dtype=torch.uint8, device="cuda")
    snaps = []
    for q in quotas:
        mb.op_linear_fwd(None, q, "bf16", T, k, n, X_, W_, None, None, Y)
        mb.op_linear_dgrad(None, q, "bf16", T, k, n, dY_, W_, None, dX)
        mb.op_linear_wgrad(None, q, "bf16", T, k, n, X_, dY_, dW, None, ws)
        torch.cuda.synchronize()
        snaps.append([bits(Y), bits(dX), bits(dW)])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b), "full-size result depends on the quota"
    return X, W, dY, Y, dX, dW


def _check_sampled(T, k, n, seed, X, W, dY, Y, dX, dW, edge_rows, edge_cols):
    rows = synth.integers(seed + 3, (32,), 0, T)
    rows[:len(edge_rows)] = edge_rows
    ridx = torch.from_numpy(rows).long().cuda()
    assert_close(from_dev(Y[ridx]), X[rows] @ W, "bf16", "Y rows")
    assert_close(from_dev(dX[ridx]), dY[rows] @ W.T, "bf16", "dX rows")
    cols = synth.integers(seed + 4, (16,), 0, n)
    cols[:len(edge_cols)] = edge_cols
    cidx = torch.from_numpy(cols).long().cuda()
    assert_close(from_dev(dW[:, cidx]), X.T @ dY[:, cols], "bf16", "dW columns")


def test_config3_decoder_output_projection_sampled(mb):
    """7B-shaped decoder of configs[2]: T = 16 x 2048 tokens, attention output projection
    4096 -> 4096 (2048 tiles of 256 x 256: eight whole rounds; the weight gradient contracts
    over 32768 tokens)."""
    T, k, n = 32768, 4096, 4096
    out = _linear_three_forms(mb, T, k, n, 9100)
    _check_sampled(T, k, n, 9100, *out, edge_rows=[0, 255, 256, T - 1], edge_cols=[0, 255, 256, n - 1])


def test_config4_vit_qkv_projection_sampled(mb):
    """6B-ViT slice of configs[3]: T = 4 x 1024 tokens, h = 3200 (12.5 tiles of 256: ragged in
    both the contraction and the output), fused QKV projection 3200 -> 9600."""
    T, k, n = 4096, 3200, 9600
    out = _linear_three_forms(mb, T, k, n, 9200)
    _check_sampled(T, k, n, 9200, *out, edge_rows=[0, 4095, 3840, 3839], edge_cols=[0, 9599, 9472, 9471])


def test_config5_audio_attention_sampled_heads(mb):
    """Audio encoder of configs[4]: B = 8, N = 1500 frames (not a multiple of the 64-row
    streamed tile nor of the 128-row workgroup tile), 20 heads of 64, full attention."""
    B, N, H, d = 8, 1500, 20, 64
    h = H * d
    qkv = quantize(synth.normal(9300, (B * N, 3 * h)), "bf16")
    dO = quantize(synth.normal(9301, (B * N, h)), "bf16")
    qkv_, dO_ = to_dev(qkv, "bf16"), to_dev(dO, "bf16")
    Oo = torch.empty((B * N, h), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    dqkv = torch.empty_like(qkv_)
    delta = torch.empty_like(lse)
    snaps = []
    for q in (256, 96):
        mb.op_attention_fwd(None, q, "bf16", B, N, H, d, 0, qkv_, Oo, lse)
        mb.op_attention_bwd(None, q, "bf16", B, N, H, d, 0, qkv_, Oo, lse, dO_, dqkv, delta)
        torch.cuda.synchronize()
        snaps.append([bits(Oo), bits(lse), bits(dqkv)])
    for a, b in zip(snaps[0], snaps[1]):
        assert np.array_equal(a, b)
    Oh, dh = from_dev(Oo), from_dev(dqkv)
    for (b, t) in ((0, 0), (7, 19), (4, 11)):
        rows = slice(b * N, (b + 1) * N)
        c = slice(t * d, (t + 1) * d)
        qh, kh, vh = qkv[rows, 0:h][:, c], qkv[rows, h:2 * h][:, c], qkv[rows, 2 * h:][:, c]
        o_ref, P = O.attention_head_fwd(qh, kh, vh, 0)
        dq, dk, dv = O.attention_head_bwd(qh, kh, vh, P, dO[rows, c])
        assert_close(Oh[rows, c], o_ref, "bf16", ("O", b, t), roundings=2)
        assert_close(dh[rows, t * d:(t + 1) * d], dq, "bf16", ("dq", b, t), roundings=8)
        assert_close(dh[rows, h + t * d:h + (t + 1) * d], dk, "bf16", ("dk", b, t), roundings=8)
        assert_close(dh[rows, 2 * h + t * d:2 * h + (t + 1) * d], dv, "bf16", ("dv", b, t), roundings=8)
