"""CPU checker ("oracle") for the forward and backward pass of the multiplexed modules.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package; only
the tests, the smoke entry and the benchmark's cpu_baseline leg call it.  It shares no
code with the HIP path.

The paper treats a module as an opaque forward+backward unit run on a quota'd stream
(Sec. 3.1 problem formulation; Sec. 4 says the engine runs stock framework modules), so
it fixes *what is scheduled*, not the layer arithmetic.  The arithmetic below is the
plain textbook definition of each layer named by the workload (ViT-style pre-LN encoder
layer, decoder layer with RMSNorm/SwiGLU/causal attention, 2-layer MLP projector, MSE),
written out with one numpy statement per mathematical step: no blocking, no fusion, no
reordering.  `@` (a library matmul) is used as a step; attention materialises the full
N x N score and probability matrices.

Precision: every function computes in the dtype of its inputs.  Tests feed float64.

Readings where the sources are silent (all recorded in the design notes as well):
  * eps = 1e-5 inside the square root for both norms; LayerNorm variance is biased.
  * GELU is the exact erf form.
  * encoder/projector linears carry biases, decoder linears carry none.
  * no positional term inside a layer; learned absolute position added by the stem.
  * multi-head attention with as many K/V heads as Q heads, scale 1/sqrt(d),
    causal mask forbids j > i, masked probability is exactly 0, no dropout.
  * loss = mean over all elements of (y - target)^2.
  * patch vector index = (c*p + i)*p + j, patches row-major over the image.
  * layer variants (not named by the workloads; offered as options): the tanh form of GELU
    (act "gelu_tanh"); rotary position embedding on q and k (cfg "rope" = base, 0 = off) in
    the original interleaved-pair form: pair i of a head, at position n of its sample, is
    rotated by the angle n * base^(-2i/d); grouped-query attention (cfg "kv_heads" < heads:
    query head t attends to key/value head t // (heads/kv_heads), w_qkv is
    [h, (heads + 2 kv_heads) d]); AdamW with decoupled weight decay and bias correction;
    a two-convolution audio stem in the style of speech encoders: Conv1d(k=3, stride 1,
    pad 1) - GELU - Conv1d(k=3, stride 2, pad 1) - GELU - learned positions, frames-major
    input [B, 2*seq, bins], weights stored [3*C_in, C_out] with row index tap*C_in + channel.

Pins (tests/test_oracle_*.py): brute-force triple-loop matmul, naive per-row softmax
attention in python loops, closed-form invariants, math.erf scalar reference, central
finite differences in float64 for every parameter tensor and the input.  There is no
value printed in the paper that a layer must reproduce, so beyond those pins the layer
arithmetic is "parity unpinned" with respect to the paper itself.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

# ----------------------------------------------------------------------------- linear


def linear_fwd(x, W, b=None):
    """Y = X W + b with W:[in,out]."""
    y = x @ W
    if b is not None:
        y = y + b
    return y


def linear_bwd(x, W, dy, has_bias=True):
    """dX = dY W^T, dW = X^T dY, db = sum over rows of dY."""
    dx = dy @ W.T
    dW = x.T @ dy
    db = dy.sum(axis=0) if has_bias else None
    return dx, dW, db


# ------------------------------------------------------------------------------ norms


def layernorm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    xhat = (x - mu) / np.sqrt(var + eps)
    return gamma * xhat + beta


def layernorm_bwd(x, gamma, dy, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    g = dy * gamma
    dx = (g - g.mean(axis=-1, keepdims=True)
          - xhat * (g * xhat).mean(axis=-1, keepdims=True)) * rstd
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    return dx, dgamma, dbeta


def rmsnorm_fwd(x, g, eps):
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    return g * x * r


def rmsnorm_bwd(x, g, dy, eps):
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    t = dy * g
    dx = r * t - (r ** 3) * x * (t * x).mean(axis=-1, keepdims=True)
    dg = (dy * x * r).sum(axis=0)
    return dx, dg


# ------------------------------------------------------------------------ activations


def gelu(z):
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + _erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def gelu_tanh(z):
    """tanh form: 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3)))."""
    return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))


def gelu_tanh_grad(z):
    t = np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3))
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * np.sqrt(2.0 / np.pi) * (1.0 + 3.0 * 0.044715 * z * z)


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def silu(z):
    return z * sigmoid(z)


def silu_grad(z):
    s = sigmoid(z)
    return s * (1.0 + z * (1.0 - s))


def swiglu_fwd(gate, up):
    return silu(gate) * up


def swiglu_bwd(gate, up, da):
    return da * up * silu_grad(gate), da * silu(gate)


# -------------------------------------------------------------------------- attention


def softmax_rows(S):
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=-1, keepdims=True)


def attention_head_fwd(q, k, v, causal):
    """One (sample, head): q,k,v [N,d] -> o [N,d], P [N,N] (materialised)."""
    N, d = q.shape
    S = (q @ k.T) / np.sqrt(float(d))
    if causal:
        S = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, S)
    P = softmax_rows(S)
    return P @ v, P


def attention_head_bwd(q, k, v, P, do):
    N, d = q.shape
    dv = P.T @ do
    dP = do @ v.T
    D = (P * dP).sum(axis=-1, keepdims=True)
    dS = P * (dP - D)
    dq = (dS @ k) / np.sqrt(float(d))
    dk = (dS.T @ q) / np.sqrt(float(d))
    return dq, dk, dv


def _split_heads(qkv, H, Hkv):
    """Column ranges of packed rows [q (H heads) | k (Hkv heads) | v (Hkv heads)]."""
    d = qkv.shape[1] // (H + 2 * Hkv)
    return d, H * d, (H + Hkv) * d


def attention_fwd(qkv, B, N, H, causal, Hkv=None):
    """qkv [B*N, (H + 2*Hkv)*d] with row = [q | k | v]; query head t owns columns t*d:(t+1)*d
    of q and attends to key/value head t // (H/Hkv) (grouped-query attention; Hkv = H is
    ordinary multi-head attention)."""
    Hkv = H if Hkv is None else Hkv
    d, ko, vo = _split_heads(qkv, H, Hkv)
    G = H // Hkv
    o = np.zeros((B * N, H * d), dtype=qkv.dtype)
    for b in range(B):
        rows = slice(b * N, (b + 1) * N)
        for t in range(H):
            u = t // G
            q = qkv[rows, t * d:(t + 1) * d]
            k = qkv[rows, ko + u * d:ko + (u + 1) * d]
            v = qkv[rows, vo + u * d:vo + (u + 1) * d]
            o[rows, t * d:(t + 1) * d], _ = attention_head_fwd(q, k, v, causal)
    return o


def attention_bwd(qkv, do, B, N, H, causal, Hkv=None):
    """Gradient of packed q|k|v; a key/value head collects the gradients of every query head
    of its group."""
    Hkv = H if Hkv is None else Hkv
    d, ko, vo = _split_heads(qkv, H, Hkv)
    G = H // Hkv
    dqkv = np.zeros_like(qkv)
    for b in range(B):
        rows = slice(b * N, (b + 1) * N)
        for t in range(H):
            u = t // G
            q = qkv[rows, t * d:(t + 1) * d]
            k = qkv[rows, ko + u * d:ko + (u + 1) * d]
            v = qkv[rows, vo + u * d:vo + (u + 1) * d]
            _, P = attention_head_fwd(q, k, v, causal)
            dq, dk, dv = attention_head_bwd(q, k, v, P, do[rows, t * d:(t + 1) * d])
            dqkv[rows, t * d:(t + 1) * d] = dq
            dqkv[rows, ko + u * d:ko + (u + 1) * d] += dk
            dqkv[rows, vo + u * d:vo + (u + 1) * d] += dv
    return dqkv


def attention_lse(qkv, B, N, H, causal, Hkv=None):
    """Row log-sum-exp of the scaled, masked scores: [B, H, N]."""
    Hkv = H if Hkv is None else Hkv
    d, ko, vo = _split_heads(qkv, H, Hkv)
    G = H // Hkv
    out = np.zeros((B, H, N), dtype=qkv.dtype)
    for b in range(B):
        rows = slice(b * N, (b + 1) * N)
        for t in range(H):
            u = t // G
            S = (qkv[rows, t * d:(t + 1) * d] @ qkv[rows, ko + u * d:ko + (u + 1) * d].T) / np.sqrt(float(d))
            if causal:
                S = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, S)
            m = S.max(axis=-1)
            out[b, t] = m + np.log(np.exp(S - m[:, None]).sum(axis=-1))
    return out


# ------------------------------------------------------------- rotary position embedding


def rope_rotate(qkv, B, N, H, base, sign=1.0, Hkv=None):
    """Rotates the q and k parts of packed [B*N, (H + 2*Hkv)*d] rows; v is left alone.  Pair
    (x[2i], x[2i+1]) of every head, in the row at position n of its sample, turns by the
    angle sign * n * base^(-2i/d).  sign = -1 is the transposed rotation, i.e. the map that
    takes gradients with respect to rotated q, k back to the unrotated ones."""
    Hkv = H if Hkv is None else Hkv
    d = qkv.shape[1] // (H + 2 * Hkv)
    out = qkv.copy()
    n = np.arange(B * N) % N
    i = np.arange(d // 2)
    ang = sign * n[:, None].astype(np.float64) * (float(base) ** (-2.0 * i / d))[None, :]
    c, s_ = np.cos(ang).astype(qkv.dtype), np.sin(ang).astype(qkv.dtype)
    for t in range(H + Hkv):                  # the q heads, then the k heads
        c0 = t * d
        xe, xo = qkv[:, c0:c0 + d:2], qkv[:, c0 + 1:c0 + d:2]
        out[:, c0:c0 + d:2] = xe * c - xo * s_
        out[:, c0 + 1:c0 + d:2] = xe * s_ + xo * c
    return out


# ------------------------------------------------------------- strided-convolution stem


def conv1d_fwd(x, w, b, stride):
    """x [B, L, C] frames-major, w [3*C, Co] (row = tap*C + channel), zero padding 1:
    y[b, t, :] = b + sum_k x[b, t*stride - 1 + k, :] @ w[k], t < L_out = (L - 1)//stride + 1."""
    B, L, C = x.shape
    Lo = (L - 1) // stride + 1
    y = np.zeros((B, Lo, w.shape[1]), dtype=x.dtype) + b
    for k in range(3):
        wk = w[k * C:(k + 1) * C]
        for t in range(Lo):
            s_ = t * stride - 1 + k
            if 0 <= s_ < L:
                y[:, t, :] += x[:, s_, :] @ wk
    return y


def conv1d_bwd(x, w, dy, stride):
    """Gradients of conv1d_fwd: (dx, dw, db)."""
    B, L, C = x.shape
    Lo = dy.shape[1]
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for k in range(3):
        wk = w[k * C:(k + 1) * C]
        for t in range(Lo):
            s_ = t * stride - 1 + k
            if 0 <= s_ < L:
                dx[:, s_, :] += dy[:, t, :] @ wk.T
                dw[k * C:(k + 1) * C] += x[:, s_, :].T @ dy[:, t, :]
    return dx, dw, dy.sum(axis=(0, 1))


def conv_stem_fwd(x, p):
    """x [B, 2*N, bins] -> [B*N, h]: conv(stride 1) - GELU - conv(stride 2) - GELU + pos[N, h]."""
    z1 = conv1d_fwd(x, p["w_c1"], p["b_c1"], 1)
    a1 = gelu(z1)
    z2 = conv1d_fwd(a1, p["w_c2"], p["b_c2"], 2)
    y = gelu(z2) + p["pos"][None, :, :]
    return y.reshape(-1, y.shape[-1]), dict(x=x, z1=z1, a1=a1, z2=z2)


def conv_stem_bwd(dy, p, s):
    g = {}
    B, N, h = s["z2"].shape
    dy = dy.reshape(B, N, h)
    g["pos"] = dy.sum(axis=0)
    dz2 = dy * gelu_grad(s["z2"])
    da1, g["w_c2"], g["b_c2"] = conv1d_bwd(s["a1"], p["w_c2"], dz2, 2)
    dz1 = da1 * gelu_grad(s["z1"])
    dx, g["w_c1"], g["b_c1"] = conv1d_bwd(s["x"], p["w_c1"], dz1, 1)
    return dx, g


# -------------------------------------------------------------------------- optimizer


def adamw_step(p, g, m, v, step, lr, beta1, beta2, eps, weight_decay):
    """One AdamW update (decoupled weight decay, bias-corrected moments); step counts from 1.
    Returns the new (p, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v


# ------------------------------------------------------------------------------- loss


def mse_fwd(y, target):
    return ((y - target) ** 2).mean()


def mse_bwd(y, target):
    return 2.0 * (y - target) / y.size


# ----------------------------------------------------------------- transformer layers
# A layer's parameters are a dict.  Encoder (LayerNorm, GELU, biases):
#   ln1_g ln1_b w_qkv b_qkv w_o b_o ln2_g ln2_b w_1 b_1 w_2 b_2
# Decoder (RMSNorm, SwiGLU, no biases):
#   rms1_g w_qkv w_o rms2_g w_gate w_up w_down


def layer_fwd(x, p, cfg):
    """One pre-norm transformer layer.  cfg: batch, seq, heads, norm, act, causal, eps."""
    B, N, H, eps = cfg["batch"], cfg["seq"], cfg["heads"], cfg["eps"]
    if cfg["norm"] == "layernorm":
        u1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    else:
        u1 = rmsnorm_fwd(x, p["rms1_g"], eps)
    qkv = linear_fwd(u1, p["w_qkv"], p.get("b_qkv"))
    Hkv = cfg.get("kv_heads") or H
    if cfg.get("rope"):
        qkv = rope_rotate(qkv, B, N, H, cfg["rope"], 1.0, Hkv)       # saved and attended in rotated form
    o = attention_fwd(qkv, B, N, H, cfg["causal"], Hkv)
    x1 = x + linear_fwd(o, p["w_o"], p.get("b_o"))
    if cfg["norm"] == "layernorm":
        u2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    else:
        u2 = rmsnorm_fwd(x1, p["rms2_g"], eps)
    if cfg["act"] in ("gelu", "gelu_tanh"):
        z = linear_fwd(u2, p["w_1"], p.get("b_1"))
        a = gelu(z) if cfg["act"] == "gelu" else gelu_tanh(z)
        y = x1 + linear_fwd(a, p["w_2"], p.get("b_2"))
        saved = dict(x=x, u1=u1, qkv=qkv, o=o, x1=x1, u2=u2, z=z, a=a)
    else:
        gate = u2 @ p["w_gate"]
        up = u2 @ p["w_up"]
        a = swiglu_fwd(gate, up)
        y = x1 + a @ p["w_down"]
        saved = dict(x=x, u1=u1, qkv=qkv, o=o, x1=x1, u2=u2, gate=gate, up=up, a=a)
    return y, saved


def layer_bwd(dy, p, s, cfg):
    """Gradients of one layer given the upstream gradient dy and the saved forward values."""
    B, N, H, eps = cfg["batch"], cfg["seq"], cfg["heads"], cfg["eps"]
    bias = bool(cfg["bias"])
    g = {}
    if cfg["act"] in ("gelu", "gelu_tanh"):
        da, g["w_2"], db2 = linear_bwd(s["a"], p["w_2"], dy, bias)
        dz = da * (gelu_grad(s["z"]) if cfg["act"] == "gelu" else gelu_tanh_grad(s["z"]))
        du2, g["w_1"], db1 = linear_bwd(s["u2"], p["w_1"], dz, bias)
        if bias:
            g["b_2"], g["b_1"] = db2, db1
    else:
        da = dy @ p["w_down"].T
        g["w_down"] = s["a"].T @ dy
        dgate, dup = swiglu_bwd(s["gate"], s["up"], da)
        g["w_gate"] = s["u2"].T @ dgate
        g["w_up"] = s["u2"].T @ dup
        du2 = dgate @ p["w_gate"].T + dup @ p["w_up"].T
    if cfg["norm"] == "layernorm":
        dn, g["ln2_g"], g["ln2_b"] = layernorm_bwd(s["x1"], p["ln2_g"], du2, eps)
    else:
        dn, g["rms2_g"] = rmsnorm_bwd(s["x1"], p["rms2_g"], du2, eps)
    dx1 = dy + dn
    do, g["w_o"], dbo = linear_bwd(s["o"], p["w_o"], dx1, bias)
    if bias:
        g["b_o"] = dbo
    Hkv = cfg.get("kv_heads") or H
    dqkv = attention_bwd(s["qkv"], do, B, N, H, cfg["causal"], Hkv)
    if cfg.get("rope"):
        dqkv = rope_rotate(dqkv, B, N, H, cfg["rope"], -1.0, Hkv)
    du1, g["w_qkv"], dbqkv = linear_bwd(s["u1"], p["w_qkv"], dqkv, bias)
    if bias:
        g["b_qkv"] = dbqkv
    if cfg["norm"] == "layernorm":
        dn, g["ln1_g"], g["ln1_b"] = layernorm_bwd(s["x"], p["ln1_g"], du1, eps)
    else:
        dn, g["rms1_g"] = rmsnorm_bwd(s["x"], p["rms1_g"], du1, eps)
    dx = dx1 + dn
    return dx, g


def stack_fwd(x, layers, cfg):
    saved = []
    for p in layers:
        x, s = layer_fwd(x, p, cfg)
        saved.append(s)
    return x, saved


def stack_bwd(dy, layers, saved, cfg):
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        dy, grads[i] = layer_bwd(dy, layers[i], saved[i], cfg)
    return dy, grads


# -------------------------------------------------------------------------- projector


def projector_fwd(x, p):
    """Linear(in->out) -> GELU -> Linear(out->out), with biases."""
    z = linear_fwd(x, p["w_1"], p["b_1"])
    a = gelu(z)
    y = linear_fwd(a, p["w_2"], p["b_2"])
    return y, dict(x=x, z=z, a=a)


def projector_bwd(dy, p, s):
    g = {}
    da, g["w_2"], g["b_2"] = linear_bwd(s["a"], p["w_2"], dy)
    dz = da * gelu_grad(s["z"])
    dx, g["w_1"], g["b_1"] = linear_bwd(s["x"], p["w_1"], dz)
    return dx, g


# ------------------------------------------------------------------------------ stems


def unfold_patches(img, patch):
    """[B,C,Hh,Ww] -> [B*nP, C*patch*patch]; vector index (c*p+i)*p+j; patches row-major."""
    B, C, Hh, Ww = img.shape
    gh, gw = Hh // patch, Ww // patch
    out = np.zeros((B * gh * gw, C * patch * patch), dtype=img.dtype)
    for b in range(B):
        for py in range(gh):
            for px in range(gw):
                blk = img[b, :, py * patch:(py + 1) * patch, px * patch:(px + 1) * patch]
                out[(b * gh + py) * gw + px] = blk.reshape(-1)
    return out


def stem_fwd(xin, p, B, N):
    """Per-token Linear(in->h) plus a learned absolute position table [N,h]."""
    y = linear_fwd(xin, p["w_stem"], p["b_stem"])
    return y + np.tile(p["pos"], (B, 1))


def stem_bwd(xin, p, dy, B, N):
    dx, dW, db = linear_bwd(xin, p["w_stem"], dy)
    dpos = dy.reshape(B, N, -1).sum(axis=0)
    return dx, dict(w_stem=dW, b_stem=db, pos=dpos)


def embedding_fwd(ids, table):
    return table[ids.reshape(-1)]


def embedding_bwd(ids, dy, vocab):
    """Plain sum over occurrences of each id."""
    dt = np.zeros((vocab, dy.shape[1]), dtype=dy.dtype)
    flat = ids.reshape(-1)
    for r in range(flat.shape[0]):
        dt[flat[r]] += dy[r]
    return dt


def concat_tokens(img_tok, txt_tok, B, n_img, n_txt):
    """Per sample: [image tokens ; text tokens] along the sequence."""
    h = img_tok.shape[1]
    out = np.zeros((B * (n_img + n_txt), h), dtype=img_tok.dtype)
    N = n_img + n_txt
    for b in range(B):
        out[b * N:b * N + n_img] = img_tok[b * n_img:(b + 1) * n_img]
        out[b * N + n_img:(b + 1) * N] = txt_tok[b * n_txt:(b + 1) * n_txt]
    return out


def split_tokens(d, B, n_img, n_txt):
    N = n_img + n_txt
    h = d.shape[1]
    di = np.zeros((B * n_img, h), dtype=d.dtype)
    dt = np.zeros((B * n_txt, h), dtype=d.dtype)
    for b in range(B):
        di[b * n_img:(b + 1) * n_img] = d[b * N:b * N + n_img]
        dt[b * n_txt:(b + 1) * n_txt] = d[b * N + n_img:(b + 1) * N]
    return di, dt


def concat_tokens_counts(img_tok, txt_rows, B, n_img, N, counts):
    """Per-sample image-token counts (reading: the workload draws them per sample while the
    sequence length stays fixed; the paper pads or truncates every module input to a uniform
    length, Sec. 3.5).  Sample b takes rows [0, counts[b]) from the first counts[b] of its n_img
    projected image tokens and rows [counts[b], N) from txt_rows, which holds one row per
    sequence position (the embedding of the id at that position)."""
    h = img_tok.shape[1]
    out = np.zeros((B * N, h), dtype=img_tok.dtype)
    for b in range(B):
        nb = int(counts[b])
        out[b * N:b * N + nb] = img_tok[b * n_img:b * n_img + nb]
        out[b * N + nb:(b + 1) * N] = txt_rows[b * N + nb:(b + 1) * N]
    return out


def split_tokens_counts(d, B, n_img, N, counts):
    """Transpose of concat_tokens_counts: image tokens that were not used and sequence
    positions that were filled by image tokens receive zero gradient."""
    h = d.shape[1]
    di = np.zeros((B * n_img, h), dtype=d.dtype)
    dt = np.zeros((B * N, h), dtype=d.dtype)
    for b in range(B):
        nb = int(counts[b])
        di[b * n_img:b * n_img + nb] = d[b * N:b * N + nb]
        dt[b * N + nb:(b + 1) * N] = d[b * N + nb:(b + 1) * N]
    return di, dt


# ------------------------------------------------------------------------------ chain


def chain_fwd_bwd(img, ids, target, P, cfgs, patch):
    """images -> unfold -> stem -> encoder -> projector -> [img;txt] -> decoder -> MSE.

    P: dict(stem, vit=[layers], proj, table, llm=[layers]); cfgs: dict(vit, llm).
    Returns loss, output, and a dict of gradients with the same structure as P.
    """
    cv, cl = cfgs["vit"], cfgs["llm"]
    B, n_img = cv["batch"], cv["seq"]
    n_txt = cl["seq"] - n_img
    patches = unfold_patches(img, patch)
    x0 = stem_fwd(patches, P["stem"], B, n_img)
    xv, sv = stack_fwd(x0, P["vit"], cv)
    xp, sp = projector_fwd(xv, P["proj"])
    xt = embedding_fwd(ids, P["table"])
    xl = concat_tokens(xp, xt, B, n_img, n_txt)
    y, sl = stack_fwd(xl, P["llm"], cl)
    loss = mse_fwd(y, target)
    dy = mse_bwd(y, target)
    dxl, gl = stack_bwd(dy, P["llm"], sl, cl)
    dxp, dxt = split_tokens(dxl, B, n_img, n_txt)
    gtab = embedding_bwd(ids, dxt, P["table"].shape[0])
    dxv, gp = projector_bwd(dxp, P["proj"], sp)
    dx0, gv = stack_bwd(dxv, P["vit"], sv, cv)
    _, gs = stem_bwd(patches, P["stem"], dx0, B, n_img)
    return loss, y, dict(stem=gs, vit=gv, proj=gp, table=gtab, llm=gl)


# ------------------------------------------------------------- stage-time definitions


def time_sliced(stage_times):
    """Iteration time under temporal multiplexing is the sum over stages (Eq. 1)."""
    return float(sum(stage_times))


def colocated(module_times):
    """A stage finishes with its slowest module (Eq. 4)."""
    return float(max(module_times))


def best_split(curves, total):
    """Exhaustive search of Eq. 4 under Eq. 5 on one GPU.

    curves: list (one per module) of dict {cu_count: time}.  Returns (quotas, time)
    minimising the max over modules subject to sum(quotas) <= total; ties are broken
    towards the lexicographically smallest quota tuple.
    """
    best = (None, float("inf"))

    def rec(i, chosen, used):
        nonlocal best
        if i == len(curves):
            t = max(curves[j][chosen[j]] for j in range(len(curves)))
            if t < best[1] or (t == best[1] and tuple(chosen) < tuple(best[0])):
                best = (list(chosen), t)
            return
        for q in sorted(curves[i]):
            if used + q <= total:
                rec(i + 1, chosen + [q], used + q)

    rec(0, [], 0)
    return best


def interference_delta(e, Bs):
    """Eq. 8: delay = e1 + e2 * sum of bandwidth utilisations + e3 * their product."""
    return e[0] + e[1] * float(np.sum(Bs)) + e[2] * float(np.prod(Bs))
