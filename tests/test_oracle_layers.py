"""Pins for whole layers, modules and the config-1 chain of the CPU checker:
identity special case, central finite differences in float64 for every parameter
tensor and the input, and a mutation check that a planted mistake is caught."""
import numpy as np
import pytest

from oracle import layers as O
from paper_2605_18710_amd import synth
from helpers import layer_params, projector_params, stem_params, small_cfg


def directional_fd(loss, params, key, R, step=1e-5):
    p_plus = dict(params); p_minus = dict(params)
    p_plus[key] = params[key] + step * R
    p_minus[key] = params[key] - step * R
    return (loss(p_plus) - loss(p_minus)) / (2 * step)


@pytest.mark.parametrize("kind", ["encoder", "decoder"])
def test_layer_is_identity_when_output_projections_are_zero(kind):
    cfg = small_cfg(kind)
    p = layer_params(cfg, 100)
    p["w_o"] = np.zeros_like(p["w_o"])
    if kind == "encoder":
        p["w_2"] = np.zeros_like(p["w_2"]); p["b_o"] = np.zeros_like(p["b_o"]); p["b_2"] = np.zeros_like(p["b_2"])
    else:
        p["w_down"] = np.zeros_like(p["w_down"])
    x = synth.normal(101, (cfg["batch"] * cfg["seq"], cfg["hidden"]))
    y, s = O.layer_fwd(x, p, cfg)
    assert np.array_equal(y, x)
    dy = synth.normal(102, x.shape)
    dx, _ = O.layer_bwd(dy, p, s, cfg)
    assert np.allclose(dx, dy, atol=1e-15)


@pytest.mark.parametrize("kind", ["encoder", "decoder"])
def test_layer_gradients_by_finite_differences(kind):
    cfg = small_cfg(kind)
    p = layer_params(cfg, 200)
    # larger weights so every path carries signal
    p = {k: (v * 10 if k.startswith("w_") else v) for k, v in p.items()}
    x = synth.normal(201, (cfg["batch"] * cfg["seq"], cfg["hidden"]))
    dy = synth.normal(202, x.shape)
    y, s = O.layer_fwd(x, p, cfg)
    dx, g = O.layer_bwd(dy, p, s, cfg)
    assert set(g) == set(p)
    for i, key in enumerate(sorted(p)):
        R = synth.normal(210 + i, p[key].shape)
        num = directional_fd(lambda q: (O.layer_fwd(x, q, cfg)[0] * dy).sum(), p, key, R)
        ana = (g[key] * R).sum()
        assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), key
    R = synth.normal(240, x.shape)
    num = ((O.layer_fwd(x + 1e-5 * R, p, cfg)[0] * dy).sum() - (O.layer_fwd(x - 1e-5 * R, p, cfg)[0] * dy).sum()) / 2e-5
    assert abs(num - (dx * R).sum()) <= 1e-6 * max(1.0, abs(num))


def test_encoder_without_positions_is_permutation_equivariant():
    cfg = small_cfg("encoder", B=1, N=6)
    p = layer_params(cfg, 300)
    x = synth.normal(301, (6, cfg["hidden"]))
    perm = np.array([4, 2, 0, 5, 1, 3])
    y, _ = O.layer_fwd(x, p, cfg)
    yp, _ = O.layer_fwd(x[perm], p, cfg)
    assert np.allclose(yp, y[perm], atol=1e-13)


def test_decoder_is_causal():
    cfg = small_cfg("decoder", B=1, N=6)
    p = layer_params(cfg, 310)
    x = synth.normal(311, (6, cfg["hidden"]))
    x2 = x.copy(); x2[4:] += 1.0
    y, _ = O.layer_fwd(x, p, cfg); y2, _ = O.layer_fwd(x2, p, cfg)
    assert np.array_equal(y[:4], y2[:4]) and not np.allclose(y[4:], y2[4:])


def test_stack_two_layers_fd():
    cfg = small_cfg("decoder")
    layers = [layer_params(cfg, 400), layer_params(cfg, 420)]
    x = synth.normal(401, (cfg["batch"] * cfg["seq"], cfg["hidden"]))
    t = synth.normal(402, x.shape)

    def loss(ls):
        return O.mse_fwd(O.stack_fwd(x, ls, cfg)[0], t)

    y, saved = O.stack_fwd(x, layers, cfg)
    dx, grads = O.stack_bwd(O.mse_bwd(y, t), layers, saved, cfg)
    for li in range(2):
        for key in ("w_qkv", "w_down", "rms1_g"):
            R = synth.normal(430 + li, layers[li][key].shape)
            lp = [dict(l) for l in layers]; lm = [dict(l) for l in layers]
            lp[li][key] = layers[li][key] + 1e-5 * R; lm[li][key] = layers[li][key] - 1e-5 * R
            num = (loss(lp) - loss(lm)) / 2e-5
            ana = (grads[li][key] * R).sum()
            assert abs(num - ana) <= 1e-6 * max(1e-3, abs(ana)), (li, key)


def test_projector_fd():
    p = projector_params(12, 20, 500)
    p = {k: (v * 10 if k.startswith("w_") else v) for k, v in p.items()}
    x = synth.normal(501, (7, 12)); dy = synth.normal(502, (7, 20))
    y, s = O.projector_fwd(x, p)
    dx, g = O.projector_bwd(dy, p, s)
    for i, key in enumerate(sorted(p)):
        R = synth.normal(510 + i, p[key].shape)
        num = directional_fd(lambda q: (O.projector_fwd(x, q)[0] * dy).sum(), p, key, R)
        assert abs(num - (g[key] * R).sum()) <= 1e-7 * max(1.0, abs(num)), key
    R = synth.normal(520, x.shape)
    num = ((O.projector_fwd(x + 1e-5 * R, p)[0] * dy).sum() - (O.projector_fwd(x - 1e-5 * R, p)[0] * dy).sum()) / 2e-5
    assert abs(num - (dx * R).sum()) <= 1e-7 * max(1.0, abs(num))


def _tiny_chain(seed=600):
    B, patch, n_img, n_txt, hv, hl = 2, 2, 4, 5, 8, 12
    cv = dict(small_cfg("encoder", B=B, N=n_img, h=hv, H=2, f=16))
    cl = dict(small_cfg("decoder", B=B, N=n_img + n_txt, h=hl, H=2, f=10))
    amp = lambda d: {k: (v * 10 if k.startswith("w_") or k in ("pos",) else v) for k, v in d.items()}
    P = dict(stem=amp(stem_params(3 * patch * patch, hv, n_img, seed + 1)),
             vit=[amp(layer_params(cv, seed + 10))],
             proj=amp(projector_params(hv, hl, seed + 40)),
             table=synth.normal(seed + 50, (7, hl)),
             llm=[amp(layer_params(cl, seed + 60))])
    img = synth.uniform(seed + 90, (B, 3, 4, 4))
    ids = synth.integers(seed + 91, (B, n_txt), 0, 7)
    target = synth.normal(seed + 92, (B * (n_img + n_txt), hl))
    return img, ids, target, P, dict(vit=cv, llm=cl), patch


def test_chain_finite_differences_every_tensor():
    img, ids, target, P, cfgs, patch = _tiny_chain()
    loss, y, G = O.chain_fwd_bwd(img, ids, target, P, cfgs, patch)
    assert loss > 0

    def perturbed(path, R, sgn):
        Q = dict(stem=dict(P["stem"]), vit=[dict(l) for l in P["vit"]], proj=dict(P["proj"]),
                 table=P["table"].copy(), llm=[dict(l) for l in P["llm"]])
        if path[0] == "table":
            Q["table"] = P["table"] + sgn * 1e-5 * R
        elif path[0] in ("vit", "llm"):
            Q[path[0]][0][path[1]] = P[path[0]][0][path[1]] + sgn * 1e-5 * R
        else:
            Q[path[0]][path[1]] = P[path[0]][path[1]] + sgn * 1e-5 * R
        return O.chain_fwd_bwd(img, ids, target, Q, cfgs, patch)[0]

    paths = [("table",)] + [("stem", k) for k in P["stem"]] + [("proj", k) for k in P["proj"]] \
        + [("vit", k) for k in P["vit"][0]] + [("llm", k) for k in P["llm"][0]]
    for i, path in enumerate(paths):
        ref = P["table"] if path[0] == "table" else (P[path[0]][0][path[1]] if path[0] in ("vit", "llm") else P[path[0]][path[1]])
        grad = G["table"] if path[0] == "table" else (G[path[0]][0][path[1]] if path[0] in ("vit", "llm") else G[path[0]][path[1]])
        R = synth.normal(700 + i, ref.shape)
        num = (perturbed(path, R, +1) - perturbed(path, R, -1)) / 2e-5
        ana = (grad * R).sum()
        assert abs(num - ana) <= 2e-6 * max(1e-4, abs(ana)), (path, num, ana)


def test_planted_mistake_is_caught(monkeypatch):
    """Mutation check of the pins themselves: drop the xhat-projection term of the
    LayerNorm backward and the finite-difference pin must fail."""
    def broken(x, gamma, dy, eps):
        mu = x.mean(-1, keepdims=True); var = ((x - mu) ** 2).mean(-1, keepdims=True)
        rstd = 1 / np.sqrt(var + eps); xhat = (x - mu) * rstd; g = dy * gamma
        return (g - g.mean(-1, keepdims=True)) * rstd, (dy * xhat).sum(0), dy.sum(0)
    monkeypatch.setattr(O, "layernorm_bwd", broken)
    with pytest.raises(AssertionError):
        test_layer_gradients_by_finite_differences("encoder")
