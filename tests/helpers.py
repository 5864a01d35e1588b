"""Shared test helpers: seeded parameter sets (numbers only, no layer arithmetic)."""
import numpy as np

from paper_2605_18710_amd import synth


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    nb = np.sqrt((b * b).sum())
    if nb == 0.0:
        return float(np.sqrt(((a - b) ** 2).sum()))
    return float(np.sqrt(((a - b) ** 2).sum()) / nb)


def elementwise_excess(got, ref, dtype, roundings=1):
    """Largest |got - ref| / bound over all elements, where the bound of an element is
    rel * |ref| + floor * rms(ref): a share of the element's own size for its last rounding and a
    share of the tensor's typical size for what the roundings before it and the fp32 summation
    order leave.  `roundings` = bf16 (or fp32) roundings between the inputs and this tensor: 1
    for a single kernel, more for a whole layer (the floor is 2^-6 per rounding for bf16: four
    times the half-ulp of a single rounding, because it has to hold for the worst of 10^5 to 10^8
    elements, not for a typical one).  A value <= 1 passes.  A tensor-wide relative L2
    norm lets a wrong 32 x 32 block of a 10^8-element tensor through; this does not: a block
    of wrong values is off by about rms(ref), tens of times the bound."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if dtype == "bf16":
        rel, floor = 2.0 ** -7, 2.0 ** -6 * (1.0 + roundings)
    else:
        rel, floor = 1e-5, 2e-5 * (1.0 + roundings)
    if rms == 0.0:
        return 0.0          # an all-zero reference: the relative-L2 check (absolute then) is the whole test
    bound = rel * np.abs(ref) + floor * rms
    return float((np.abs(got - ref) / bound).max())


def assert_close(got, ref, dtype, what="", roundings=1, l2=None):
    """The stated tolerance (relative L2) and the element-by-element bound, together."""
    e = rel_l2(got, ref)
    assert e <= (tol(dtype) if l2 is None else l2), (what, "rel L2", e)
    x = elementwise_excess(got, ref, dtype, roundings)
    assert x <= 1.0, (what, "element beyond its bound by a factor of", x)


def fast_layer_params(cfg, seed):
    """Layer parameters for full-size shapes: matrices uniform with standard deviation 0.02 from
    the bulk generator (the counter-based normal generator needs seconds per 10^7 values on the
    host; these hold 10^8), gains and biases perturbed like layer_params."""
    h, f = cfg["hidden"], cfg["mlp"]
    s = iter(range(seed, seed + 64))
    a = 0.02 * np.sqrt(3.0)
    n = lambda shape: synth.bulk_uniform(next(s), shape, -a, a)
    one = lambda k: 1.0 + synth.normal(next(s), (k,), 0.0, 0.02)
    zero = lambda k: synth.normal(next(s), (k,), 0.0, 0.02)
    if cfg["kind"] == "encoder":
        return dict(ln1_g=one(h), ln1_b=zero(h), w_qkv=n((h, 3 * h)), b_qkv=zero(3 * h),
                    w_o=n((h, h)), b_o=zero(h), ln2_g=one(h), ln2_b=zero(h),
                    w_1=n((h, f)), b_1=zero(f), w_2=n((f, h)), b_2=zero(h))
    return dict(rms1_g=one(h), w_qkv=n((h, 3 * h)), w_o=n((h, h)), rms2_g=one(h),
                w_gate=n((h, f)), w_up=n((h, f)), w_down=n((f, h)))


def layer_params(cfg, seed, perturb=True):
    """N(0,0.02) matrices; norm gains 1 and biases 0, perturbed by N(0,0.02) when asked
    so that their gradients are exercised."""
    h, f = cfg["hidden"], cfg["mlp"]
    s = iter(range(seed, seed + 64))
    n = lambda shape: synth.normal(next(s), shape, 0.0, 0.02)
    one = lambda k: 1.0 + (n((k,)) if perturb else 0.0)
    zero = lambda k: (n((k,)) if perturb else np.zeros(k))
    if cfg["kind"] == "encoder":
        return dict(ln1_g=one(h), ln1_b=zero(h), w_qkv=n((h, 3 * h)), b_qkv=zero(3 * h),
                    w_o=n((h, h)), b_o=zero(h), ln2_g=one(h), ln2_b=zero(h),
                    w_1=n((h, f)), b_1=zero(f), w_2=n((f, h)), b_2=zero(h))
    return dict(rms1_g=one(h), w_qkv=n((h, 3 * h)), w_o=n((h, h)), rms2_g=one(h),
                w_gate=n((h, f)), w_up=n((h, f)), w_down=n((f, h)))


def projector_params(din, dout, seed, perturb=True):
    s = iter(range(seed, seed + 8))
    n = lambda shape: synth.normal(next(s), shape, 0.0, 0.02)
    zero = lambda k: (n((k,)) if perturb else np.zeros(k))
    return dict(w_1=n((din, dout)), b_1=zero(dout), w_2=n((dout, dout)), b_2=zero(dout))


def stem_params(din, h, N, seed, perturb=True):
    s = iter(range(seed, seed + 8))
    n = lambda shape: synth.normal(next(s), shape, 0.0, 0.02)
    return dict(w_stem=n((din, h)), b_stem=(n((h,)) if perturb else np.zeros(h)), pos=n((N, h)))


def small_cfg(kind, B=2, N=8, h=16, H=2, f=24):
    if kind == "encoder":
        return dict(kind="encoder", batch=B, seq=N, hidden=h, heads=H, mlp=f, layers=1,
                    norm="layernorm", act="gelu", causal=0, bias=1, eps=1e-5)
    return dict(kind="decoder", batch=B, seq=N, hidden=h, heads=H, mlp=f, layers=1,
                norm="rmsnorm", act="swiglu", causal=1, bias=0, eps=1e-5)


# ------------------------------------------------------------------ GPU-side helpers
def quantize(a, dtype):
    """What the GPU will see: values rounded to the storage dtype, as float64."""
    if dtype == "bf16":
        return synth.round_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def quantize_tree(t, dtype):
    if isinstance(t, dict):
        return {k: quantize_tree(v, dtype) for k, v in t.items()}
    if isinstance(t, list):
        return [quantize_tree(v, dtype) for v in t]
    return quantize(t, dtype)


def to_dev(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda().contiguous()


def from_dev(t):
    return t.float().cpu().numpy().astype(np.float64)


def tol(dtype):
    """Relative L2 bound: 1e-5 on the fp32 path, 2e-2 for bf16 storage with fp32
    accumulation (the workload's stated tolerances)."""
    return 2e-2 if dtype == "bf16" else 1e-5


def load_layer_params(module, layers):
    """Copy oracle-style per-layer dicts into a module's flat parameter buffer."""
    for l, p in enumerate(layers):
        for k, v in p.items():
            if k in ("w_gate", "w_up"):
                continue
            module.set_tensor(f"L{l}.{k}", v)
        if "w_gate" in p:
            module.set_tensor(f"L{l}.w_gu", np.concatenate([p["w_gate"], p["w_up"]], axis=1))


def read_layer_grads(module, layers):
    out = []
    for l, p in enumerate(layers):
        g = {}
        for k in p:
            if k in ("w_gate", "w_up"):
                continue
            g[k] = module.get_tensor(f"L{l}.{k}", grads=True).reshape(np.shape(p[k]))
        if "w_gate" in p:
            gu = module.get_tensor(f"L{l}.w_gu", grads=True)
            f = p["w_gate"].shape[1]
            g["w_gate"], g["w_up"] = gu[:, :f], gu[:, f:]
        out.append(g)
    return out


def load_flat_params(module, p):
    for k, v in p.items():
        module.set_tensor(k, v)


def read_flat_grads(module, p):
    return {k: module.get_tensor(k, grads=True).reshape(np.shape(v)) for k, v in p.items()}
