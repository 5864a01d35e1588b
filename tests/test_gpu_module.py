"""Module-level parity through the C ABI: forward output, input gradient and every
parameter gradient of encoder / decoder / projector / stem modules against the CPU
checker, bit-identity across quotas, and the chained config-1 stage end to end."""
import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import (assert_close, rel_l2, quantize, quantize_tree, to_dev, from_dev, tol, layer_params, projector_params,
                     stem_params, load_layer_params, read_layer_grads, load_flat_params, read_flat_grads)

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


def enc(B, N, h, H, f, L):
    return dict(kind="encoder", batch=B, seq=N, hidden=h, heads=H, mlp=f, layers=L,
                norm="layernorm", act="gelu", causal=0, bias=1, eps=1e-5)


def dec(B, N, h, H, f, L):
    return dict(kind="decoder", batch=B, seq=N, hidden=h, heads=H, mlp=f, layers=L,
                norm="rmsnorm", act="swiglu", causal=1, bias=0, eps=1e-5)


STACKS = [
    ("f32", enc(2, 16, 128, 4, 512, 1)),        # config-1 vision layer
    ("f32", dec(2, 128, 128, 4, 384, 1)),       # config-1 decoder layer
    ("f32", dec(1, 24, 64, 2, 96, 3)),
    ("bf16", enc(2, 196, 256, 4, 1024, 2)),     # ragged T = 392, head 64
    ("bf16", dec(2, 160, 512, 4, 768, 2)),      # head 128, causal
]


@pytest.mark.parametrize("dtype,cfg", STACKS)
def test_stack_step_matches_oracle_and_is_quota_invariant(mb, dtype, cfg):
    T, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
    layers = quantize_tree([layer_params(cfg, 1000 + 100 * l) for l in range(cfg["layers"])], dtype)
    x = quantize(synth.normal(2000, (T, h)), dtype)
    target = quantize(synth.normal(2001, (T, h)), dtype)
    y_ref, saved = O.stack_fwd(x, layers, cfg)
    loss_ref = O.mse_fwd(y_ref, target)
    dx_ref, g_ref = O.stack_bwd(O.mse_bwd(y_ref, target), layers, saved, cfg)

    m = mb.Module(cfg, dtype)
    load_layer_params(m, layers)
    x_, t_ = to_dev(x, dtype), to_dev(target, dtype)
    first = None
    for q in (256, 96, 17):
        y = torch.empty_like(x_); dx = torch.empty_like(x_)
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        m.grads.zero_()
        m.step(q, None, x_, y, target=t_, dx=dx, loss=loss)
        torch.cuda.synchronize()
        snap = [bits(y), bits(dx), bits(m.grads), bits(loss)]
        if first is None:
            first = snap
            nl = cfg["layers"]
            assert_close(from_dev(y), y_ref, dtype, "y", roundings=8 * nl)
            assert abs(loss.item() - loss_ref) <= tol(dtype) * loss_ref
            assert_close(from_dev(dx), dx_ref, dtype, "dx", roundings=24 * nl)
            g = read_layer_grads(m, layers)
            for l in range(nl):
                for k in g_ref[l]:
                    assert_close(g[l][k], g_ref[l][k], dtype, (l, k), roundings=24 * nl)
        else:
            for a, b in zip(snap, first):
                assert np.array_equal(a, b), "module step depends on the quota"
    m.destroy()


def test_given_upstream_gradient_instead_of_target(mb):
    cfg = dec(1, 32, 64, 2, 96, 1)
    layers = quantize_tree([layer_params(cfg, 3000)], "f32")
    x = quantize(synth.normal(3001, (32, 64)), "f32"); dy = quantize(synth.normal(3002, (32, 64)), "f32")
    y_ref, saved = O.stack_fwd(x, layers, cfg)
    dx_ref, g_ref = O.stack_bwd(dy, layers, saved, cfg)
    m = mb.Module(cfg, "f32")
    load_layer_params(m, layers)
    x_, dy_ = to_dev(x, "f32"), to_dev(dy, "f32")
    y = torch.empty_like(x_); dx = torch.empty_like(x_)
    m.step(256, None, x_, y, dy=dy_, dx=dx)
    torch.cuda.synchronize()
    assert rel_l2(from_dev(dx), dx_ref) <= 1e-5
    assert rel_l2(read_layer_grads(m, layers)[0]["w_qkv"], g_ref[0]["w_qkv"]) <= 1e-5
    with pytest.raises(mb.MosaicError):
        m.step(256, None, x_, y, dx=dx)                 # neither dy nor target
    with pytest.raises(mb.MosaicError):
        m.step(300, None, x_, y, dy=dy_, dx=dx)         # quota beyond the device
    m.destroy()


@pytest.mark.parametrize("dtype,T,din,dout", [("f32", 32, 128, 128), ("bf16", 392, 256, 512)])
def test_projector(mb, dtype, T, din, dout):
    cfg = dict(kind="projector", batch=1, seq=T, in_dim=din, out_dim=dout)
    p = quantize_tree(projector_params(din, dout, 4000), dtype)
    x = quantize(synth.normal(4001, (T, din)), dtype); dy = quantize(synth.normal(4002, (T, dout)), dtype)
    y_ref, s = O.projector_fwd(x, p)
    dx_ref, g_ref = O.projector_bwd(dy, p, s)
    m = mb.Module(cfg, dtype)
    load_flat_params(m, p)
    x_, dy_ = to_dev(x, dtype), to_dev(dy, dtype)
    y = torch.empty((T, dout), dtype=x_.dtype, device="cuda"); dx = torch.empty_like(x_)
    m.step(256, None, x_, y, dy=dy_, dx=dx)
    torch.cuda.synchronize()
    assert rel_l2(from_dev(y), y_ref) <= tol(dtype)
    assert rel_l2(from_dev(dx), dx_ref) <= tol(dtype)
    g = read_flat_grads(m, p)
    for k in g_ref:
        assert rel_l2(g[k], g_ref[k]) <= tol(dtype), k
    m.destroy()


def build_config1(mb, dtype="f32"):
    """The tiny 2-module stage as a chain of five library modules."""
    wl = synth.WORKLOADS[0]
    cv, cp, cl = wl["modules"]
    B, n_img, hv, hl = cv["batch"], cv["seq"], cv["hidden"], cl["hidden"]
    n_txt = cl["seq"] - n_img
    seed = synth.tensor_seed(0, 0)
    P = dict(stem=stem_params(cv["in_dim"], hv, n_img, seed + 100),
             vit=[layer_params(cv, seed + 200)], proj=projector_params(hv, hl, seed + 300),
             table=synth.normal(seed + 400, (cl["vocab"], hl), 0, 0.02), llm=[layer_params(cl, seed + 500)])
    P = quantize_tree(P, dtype)
    img = quantize(synth.uniform(seed + 1, wl["image"]), dtype)
    ids = synth.integers(seed + 2, (B, n_txt), 0, cl["vocab"])
    target = quantize(synth.normal(seed + 3, (B * cl["seq"], hl)), dtype)
    mods = [
        mb.Module(dict(kind="patch_stem", batch=B, seq=n_img, hidden=hv, in_dim=cv["in_dim"], patch=wl["patch"]), dtype),
        mb.Module(cv, dtype),
        mb.Module(dict(cp), dtype),
        mb.Module(dict(kind="text_stem", batch=B, seq=cl["seq"], hidden=hl, vocab=cl["vocab"], n_img=n_img), dtype),
        mb.Module(cl, dtype),
    ]
    load_flat_params(mods[0], P["stem"]); load_layer_params(mods[1], P["vit"]); load_flat_params(mods[2], P["proj"])
    mods[3].set_tensor("table", P["table"]); load_layer_params(mods[4], P["llm"])
    ids_ = torch.from_numpy(ids.reshape(-1)).cuda()
    mods[3].bind_ids(ids_)
    return wl, P, img, ids, target, mods, ids_


def test_config1_chain_end_to_end(mb):
    dtype = "f32"
    wl, P, img, ids, target, mods, ids_ = build_config1(mb, dtype)
    cv, cp, cl = wl["modules"]
    loss_ref, y_ref, G = O.chain_fwd_bwd(img, ids, target, P, dict(vit=cv, llm=cl), wl["patch"])
    td = torch.float32
    x0 = to_dev(img, dtype)
    ys = [torch.empty(m.out_elems, dtype=td, device="cuda") for m in mods]
    dxs = [None] + [torch.empty(m.in_elems, dtype=td, device="cuda") for m in mods[1:]]
    xs = [x0] + ys[:-1]
    dys = dxs[1:] + [None]
    t_ = to_dev(target, dtype)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    mb.pool_reserve(256, 0, mb.STRIPED)
    r = mb.stage_run(mods, xs, ys, [256] * 5, [0] * 5, mb.STRIPED, mb.CHAINED, dy=dys,
                     target=[None] * 4 + [t_], dx=dxs, loss=[None] * 4 + [loss])
    assert r["stage_ms"] > 0
    assert rel_l2(from_dev(ys[-1]).reshape(y_ref.shape), y_ref) <= 1e-5
    assert abs(loss.item() - loss_ref) <= 1e-5 * loss_ref
    checks = [(read_flat_grads(mods[0], P["stem"]), G["stem"]), (read_layer_grads(mods[1], P["vit"])[0], G["vit"][0]),
              (read_flat_grads(mods[2], P["proj"]), G["proj"]), (read_layer_grads(mods[4], P["llm"])[0], G["llm"][0])]
    for got, ref in checks:
        for k in ref:
            assert rel_l2(got[k], ref[k]) <= 1e-5, k
    assert rel_l2(mods[3].get_tensor("table", grads=True), G["table"]) <= 1e-5
    for m in mods:
        m.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_text_stem_with_per_sample_image_token_counts_chained(mb, dtype):
    """Fixed sequence length, a different number of image tokens per sample (the mix of the
    large-encoder / mid-LLM workload at reduced size): text stem -> decoder layer -> loss as a
    chained stage; output, loss, the gradient of the image tokens (zero rows where a sample did
    not use a token), the embedding-table gradient and the decoder's gradients against the
    checker.  One count is 0 and one is n_img; one id lies outside the table (clamped both ways)."""
    B, n_img, N, h, vocab = 4, 24, 64, 64, 50
    cl = dec(B, N, h, 2, 96, 1)
    seed = 880
    counts = synth.integers(seed, (B,), 6, n_img + 1)
    counts[0], counts[1] = 0, n_img
    ids = synth.integers(seed + 1, (B, N), 0, vocab)
    ids[2, N - 1] = vocab + 7                                   # outside the table: reads and updates the last row
    ids_ref = np.clip(ids, 0, vocab - 1)
    table = quantize(synth.normal(seed + 2, (vocab, h), 0, 0.02), dtype)
    img = quantize(synth.normal(seed + 3, (B * n_img, h)), dtype)
    target = quantize(synth.normal(seed + 4, (B * N, h)), dtype)
    layers = quantize_tree([layer_params(cl, seed + 10)], dtype)
    x_ref = O.concat_tokens_counts(img, O.embedding_fwd(ids_ref, table), B, n_img, N, counts)
    y_ref, saved = O.stack_fwd(x_ref, layers, cl)
    loss_ref = O.mse_fwd(y_ref, target)
    dxl, g_ref = O.stack_bwd(O.mse_bwd(y_ref, target), layers, saved, cl)
    dimg_ref, dtxt = O.split_tokens_counts(dxl, B, n_img, N, counts)
    gtab_ref = O.embedding_bwd(ids_ref, dtxt, vocab)

    stem = mb.Module(dict(kind="text_stem", batch=B, seq=N, hidden=h, vocab=vocab, n_img=n_img), dtype)
    llm = mb.Module(cl, dtype)
    try:
        stem.set_tensor("table", table); load_layer_params(llm, layers)
        ids_ = torch.from_numpy(ids.reshape(-1)).cuda(); counts_ = torch.from_numpy(counts).cuda()
        stem.bind_ids(ids_); stem.bind_image_counts(counts_)
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        x0 = to_dev(img, dtype)
        ys = [torch.empty(B * N * h, dtype=td, device="cuda") for _ in range(2)]
        dxs = [torch.full((B * n_img * h,), 7.0, dtype=td, device="cuda"), torch.empty(B * N * h, dtype=td, device="cuda")]
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        mb.pool_reserve(256, 0, mb.STRIPED)
        mb.stage_run([stem, llm], [x0, ys[0]], ys, [256, 256], [0, 0], mb.STRIPED, mb.CHAINED, dy=[dxs[1], None],
                     target=[None, to_dev(target, dtype)], dx=dxs, loss=[None, loss])
        assert np.array_equal(from_dev(ys[0]).reshape(B * N, h), x_ref), "sequence assembly is a copy: exact"
        assert rel_l2(from_dev(ys[1]).reshape(B * N, h), y_ref) <= tol(dtype)
        assert abs(loss.item() - loss_ref) <= tol(dtype) * loss_ref
        dimg = from_dev(dxs[0]).reshape(B * n_img, h)
        assert rel_l2(dimg, dimg_ref) <= tol(dtype)
        for b in range(B):
            assert not dimg[b * n_img + counts[b]:(b + 1) * n_img].any(), "unused image tokens must get zero gradient"
        assert rel_l2(stem.get_tensor("table", grads=True), gtab_ref) <= tol(dtype)
        g = read_layer_grads(llm, layers)[0]
        for k in g_ref[0]:
            assert rel_l2(g[k], g_ref[0][k]) <= tol(dtype), k
    finally:
        stem.destroy(); llm.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_embedding_gradient_with_heavily_repeated_ids(mb, dtype):
    """A table of five rows under 3 x 1096 text positions, two thirds of them the same id: the
    owner of that row gathers its occurrences through several fills of its position list; one
    row is never used (zero gradient), ids outside the table count for the nearest row.  Rows
    of 520 elements span three column blocks, the last one ragged.  Bit-identical across quotas."""
    B, n_img, N, h, vocab = 3, 4, 1100, 520, 5
    seed = 990
    ids = synth.integers(seed, (B, N - n_img), 0, 3)                 # ids 0..2; row 3 stays unused
    heavy = synth.uniform(seed + 1, (B, N - n_img), 0.0, 1.0) < 0.66
    ids[heavy] = 2
    ids[1, 17] = -3; ids[2, 900] = vocab + 11                         # clamped to rows 0 and 4
    ids_ref = np.clip(ids, 0, vocab - 1)
    dy = quantize(synth.normal(seed + 2, (B * N, h)), dtype)
    img = quantize(synth.normal(seed + 3, (B * n_img, h)), dtype)
    table = quantize(synth.normal(seed + 4, (vocab, h), 0, 0.02), dtype)
    dimg_ref, dtxt = O.split_tokens(dy, B, n_img, N - n_img)
    gtab_ref = O.embedding_bwd(ids_ref, dtxt, vocab)
    assert (ids_ref == 2).sum() > 2 * 1024 and not (ids_ref == 3).any()
    stem = mb.Module(dict(kind="text_stem", batch=B, seq=N, hidden=h, vocab=vocab, n_img=n_img), dtype)
    try:
        stem.set_tensor("table", table)
        ids_ = torch.from_numpy(ids.reshape(-1).astype(np.int32)).cuda()
        stem.bind_ids(ids_)
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        y = torch.empty(B * N * h, dtype=td, device="cuda")
        snaps = []
        for quota in (256, 24):
            stem.grads.fill_(float("nan"))
            dx = torch.full((B * n_img * h,), float("nan"), dtype=td, device="cuda")
            stem.step(quota, None, to_dev(img, dtype), y, dy=to_dev(dy, dtype), dx=dx)
            torch.cuda.synchronize()
            snaps.append((stem.grads.clone(), dx.clone()))
        got = stem.get_tensor("table", grads=True)
        # a row's gradient is a sum over up to 2200 rounded rows: rounding of the result plus fp32 accumulation
        assert_close(got, gtab_ref, dtype, "table gradient", roundings=4)
        assert not got[3].any(), "a row nobody uses gets a zero gradient"
        assert np.array_equal(from_dev(snaps[0][1]).reshape(B * n_img, h), dimg_ref), "image-token gradient is a copy: exact"
        for a, b in zip(snaps[0], snaps[1]):
            assert torch.equal(a.view(torch.int32 if dtype == "f32" else torch.int16), b.view(torch.int32 if dtype == "f32" else torch.int16))
    finally:
        stem.destroy()

