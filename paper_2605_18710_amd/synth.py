"""Seeded synthetic inputs for the multiplexed-stage workloads.

A counter-based generator: element i of a tensor with seed s is a pure function of
(s, i), so the CPU checker and the GPU path consume identical bits regardless of the
order or chunking in which tensors are produced.  This module holds no layer
arithmetic; it only draws numbers and describes workload shapes.

The paper trains on mock data of uniform per-modality sizes (Sec. 5.1, Table 2); the
shapes below are the synthetic stand-ins for those workloads.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def tensor_seed(config: int, tensor_id: int) -> int:
    """Seed convention: 18710*1000 + 10*config + tensor_id (tensor_id may exceed 9)."""
    return 18710 * 1000 + 10 * config + tensor_id


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser applied to a uint64 counter array (published algorithm)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _bits(seed: int, n: int, stream: int = 0, start: int = 0) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = _splitmix64(np.array([seed], dtype=np.uint64) * np.uint64(2) + np.uint64(stream))[0]
        ctr = np.arange(start, start + n, dtype=np.uint64) + base
    return _splitmix64(ctr)


def uniform(seed: int, shape, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    """float64 uniform in [lo, hi) with 53 random mantissa bits."""
    n = int(np.prod(shape, dtype=np.int64))
    u = (_bits(seed, n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return (lo + (hi - lo) * u).reshape(shape)


def normal(seed: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """float64 normal by Box-Muller over two independent counter streams."""
    n = int(np.prod(shape, dtype=np.int64))
    u1 = ((_bits(seed, n, 0) >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / (1 << 53))
    u2 = (_bits(seed, n, 1) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + std * z).reshape(shape)


def normal_range(seed: int, start: int, end: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Elements [start, end) of the flat stream that normal(seed, ...) draws from."""
    n = end - start
    u1 = ((_bits(seed, n, 0, start) >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / (1 << 53))
    u2 = (_bits(seed, n, 1, start) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return mean + std * (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2))


def bulk_uniform(seed: int, shape, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    """float64 uniform in [lo, hi) for tensors of 10^8 elements and more (full-size weights in
    tests), from numpy's PCG64 stream seeded with `seed`: deterministic like the counter-based
    draws above, without their element-addressability, and fifty times faster."""
    g = np.random.Generator(np.random.PCG64(seed))
    u = g.random(size=shape, dtype=np.float32).astype(np.float64)
    return lo + (hi - lo) * u


def integers(seed: int, shape, lo: int, hi: int) -> np.ndarray:
    """int32 uniform in [lo, hi)."""
    n = int(np.prod(shape, dtype=np.int64))
    r = _bits(seed, n) % np.uint64(hi - lo)
    return (r.astype(np.int64) + lo).astype(np.int32).reshape(shape)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returned as float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(f.shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of round_bf16(x)."""
    return (round_bf16(x).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# Workload shapes.  kind: "encoder" (pre-LN, LayerNorm, GELU, biases, full attention),
# "decoder" (RMSNorm, SwiGLU, no biases, causal attention), "projector" (2-layer MLP).
# --------------------------------------------------------------------------------------

def _enc(name, B, N, h, H, f, L, stem_in=0):
    return dict(name=name, kind="encoder", batch=B, seq=N, hidden=h, heads=H, mlp=f,
                layers=L, norm="layernorm", act="gelu", causal=0, bias=1, eps=1e-5,
                in_dim=stem_in, out_dim=h)


def _dec(name, B, N, h, H, f, L, vocab=0, n_img=0):
    return dict(name=name, kind="decoder", batch=B, seq=N, hidden=h, heads=H, mlp=f,
                layers=L, norm="rmsnorm", act="swiglu", causal=1, bias=0, eps=1e-5,
                in_dim=0, out_dim=h, vocab=vocab, n_img=n_img)


def _proj(name, B, N, din, dout):
    return dict(name=name, kind="projector", batch=B, seq=N, hidden=dout, heads=0, mlp=0,
                layers=1, norm="none", act="gelu", causal=0, bias=1, eps=0.0,
                in_dim=din, out_dim=dout)


WORKLOADS = {
    # config index -> dict(dtype, modules, quota plans in CUs, which modules hold a quota)
    0: dict(name="tiny-fp32", dtype="f32",
            modules=[_enc("vit", 2, 16, 128, 4, 512, 1, stem_in=768),
                     _proj("proj", 2, 16, 128, 128),
                     _dec("llm", 2, 128, 128, 4, 384, 1, vocab=1000, n_img=16)],
            groups=[["vit", "proj"], ["llm"]], plans=[[128, 128]],
            image=(2, 3, 64, 64), patch=16),
    1: dict(name="clipb-smalllm-bf16", dtype="bf16",
            modules=[_enc("vit", 8, 196, 768, 12, 3072, 12, stem_in=768),
                     _proj("proj", 8, 196, 768, 2048),
                     _dec("llm", 8, 1024, 2048, 16, 5632, 4, vocab=32000, n_img=196)],
            groups=[["vit", "proj"], ["llm"]],
            plans=[[64, 192], [96, 160], [128, 128], [160, 96], [192, 64]],
            image=(8, 3, 224, 224), patch=16),
    2: dict(name="vitl-7b-bf16", dtype="bf16",
            modules=[_enc("vit", 16, 576, 1024, 16, 4096, 24, stem_in=588),
                     _dec("llm", 16, 2048, 4096, 32, 11008, 4)],
            groups=[["vit"], ["llm"]], plans=[[32, 224], [64, 192]],
            image=(16, 3, 336, 336), patch=14),
    3: dict(name="vit6b-20b-bf16", dtype="bf16",
            modules=[_enc("vit", 4, 1024, 3200, 25, 12800, 8, stem_in=588),
                     _proj("proj", 4, 1024, 3200, 5120),
                     _dec("llm", 4, 4096, 5120, 40, 13824, 4)],
            groups=[["vit", "proj"], ["llm"]], plans=[[32, 224], [64, 192]],
            image=(4, 3, 448, 448), patch=14),
    4: dict(name="vision-audio-llm-bf16", dtype="bf16",
            modules=[_enc("vit", 8, 576, 1024, 16, 4096, 12, stem_in=588),
                     _enc("audio", 8, 1500, 1280, 20, 5120, 8, stem_in=80),
                     _dec("llm", 8, 4096, 4096, 32, 11008, 4)],
            groups=[["vit"], ["audio"], ["llm"]],
            plans=[[32, 32, 192], [32, 64, 160], [64, 64, 128], [32, 96, 128], [64, 32, 160]],
            image=(8, 3, 336, 336), patch=14),
}


def module_flops(m: dict) -> float:
    """Model FLOPs of one forward+backward step (backward = 2x forward, no recompute)."""
    T = m["batch"] * m["seq"]
    if m["kind"] == "projector":
        return 3.0 * 2.0 * T * (m["in_dim"] * m["out_dim"] + m["out_dim"] * m["out_dim"])
    h, f, N, B = m["hidden"], m["mlp"], m["seq"], m["batch"]
    gemm = 8.0 * T * h * h + (6.0 if m["act"] == "swiglu" else 4.0) * T * h * f
    attn = 4.0 * B * N * N * h * (0.5 if m["causal"] else 1.0)
    return 3.0 * m["layers"] * (gemm + attn)


def module_bytes(m: dict, elem: int = 2) -> float:
    """Algorithmic HBM bytes of one forward+backward step: every kernel reads its operands and
    writes its result once (GEMM: the three matrices; attention: packed q|k|v, output and
    their gradients; norms, activations and residuals: one pass per tensor).  Used as the
    numerator of the bandwidth-utilisation proxy B(m, a) = bytes / (time x peak)."""
    T = m["batch"] * m["seq"]

    def gemm3(k, n):          # forward, input-gradient and weight-gradient forms of one linear layer
        one = T * k + k * n + T * n
        return 3.0 * one

    if m["kind"] == "projector":
        d_in, d_out = m["in_dim"], m["out_dim"]
        return elem * (gemm3(d_in, d_out) + gemm3(d_out, d_out) + 5.0 * T * d_out)
    h, f = m["hidden"], m["mlp"]
    zf = 2 * f if m["act"] == "swiglu" else f
    gemms = gemm3(h, 3 * h) + gemm3(h, h) + gemm3(h, zf) + gemm3(f, h) + 2.0 * T * h      # + two residual reads
    attn = 4.0 * T * h + 8.0 * T * h                      # fwd: q|k|v in, O out; bwd: q|k|v, O, dO in, dq|dk|dv out
    norms = 2 * (2.0 * T * h) + 2 * (4.0 * T * h + 2.0 * T * h)
    act = (3.0 + 5.0) * T * f if m["act"] == "swiglu" else (2.0 + 3.0) * T * f
    return elem * m["layers"] * (gemms + attn + norms + act)
