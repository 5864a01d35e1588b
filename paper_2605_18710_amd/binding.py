"""Thin ctypes binding of libmosaic.so (the C ABI declared in include/mosaic.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch is used for device memory (tensors whose data_ptr() is handed over) and nothing
else.  There is no fallback: if the library is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmosaic.so")

OK, EINVAL, EQUOTA, ENOMEM, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
ENCODER, DECODER, PROJECTOR, PATCH_STEM, TEXT_STEM, CONV_STEM = 0, 1, 2, 3, 4, 5
NORM_NONE, LAYERNORM, RMSNORM = 0, 1, 2
GELU, SWIGLU = 0, 1
STRIPED, XCD_ALIGNED = 0, 1
COLOCATED, TIME_SLICED, CHAINED = 0, 1, 2
MAX_STAGE_MODULES = 8

_KIND = {"encoder": ENCODER, "decoder": DECODER, "projector": PROJECTOR,
         "patch_stem": PATCH_STEM, "text_stem": TEXT_STEM, "conv_stem": CONV_STEM}
_NORM = {"none": NORM_NONE, "layernorm": LAYERNORM, "rmsnorm": RMSNORM}
GELU_TANH = 2
_ACT = {"gelu": GELU, "swiglu": SWIGLU, "gelu_tanh": GELU_TANH}
_DTYPE = {"f32": F32, "bf16": BF16}


class MosaicError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"mosaic status {status}: {message}")
        self.status = status


class ModuleDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32),
                ("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32),
                ("mlp", C.c_int32), ("batch", C.c_int32), ("seq", C.c_int32),
                ("norm", C.c_int32), ("act", C.c_int32), ("causal", C.c_int32), ("bias", C.c_int32),
                ("eps", C.c_float),
                ("in_dim", C.c_int32), ("out_dim", C.c_int32),
                ("vocab", C.c_int32), ("n_img", C.c_int32), ("patch", C.c_int32),
                ("rope_base", C.c_float), ("kv_heads", C.c_int32)]


class Stage(C.Structure):
    _fields_ = [("n", C.c_int32), ("modules", C.POINTER(C.c_void_p)),
                ("x", C.POINTER(C.c_void_p)), ("dy", C.POINTER(C.c_void_p)),
                ("target", C.POINTER(C.c_void_p)), ("y", C.POINTER(C.c_void_p)),
                ("dx", C.POINTER(C.c_void_p)), ("loss", C.POINTER(C.c_void_p))]


class Plan(C.Structure):
    _fields_ = [("n", C.c_int32), ("cu_quota", C.POINTER(C.c_int32)),
                ("cu_offset", C.POINTER(C.c_int32)), ("layout", C.c_int32), ("mode", C.c_int32)]


class Timing(C.Structure):
    _fields_ = [("stage_ms", C.c_float), ("module_ms", C.c_float * MAX_STAGE_MODULES)]


# name -> (restype, argtypes); mirrors include/mosaic.h one to one
_vp, _i32, _i64, _f32, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
SIGNATURES = {
    "mosaic_last_error": (C.c_char_p, []),
    "mosaic_device_cu_count": (_i32, []),
    "mosaic_device_xcd_count": (_i32, []),
    "mosaic_cu_mask_build": (_i32, [_i32, _i32, _i32, _i32, _i32, C.POINTER(C.c_uint32), _i32]),
    "mosaic_stream_create": (_i32, [_i32, _i32, _i32, C.POINTER(_vp)]),
    "mosaic_stream_native": (_vp, [_vp]),
    "mosaic_stream_quota": (_i32, [_vp]),
    "mosaic_stream_offset": (_i32, [_vp]),
    "mosaic_stream_destroy": (_i32, [_vp]),
    "mosaic_interference_delta": (C.c_double, [C.POINTER(C.c_double), _i32, C.POINTER(C.c_double)]),
    "mosaic_interference_fit": (_i32, [_i32, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double), _i32,
                                       C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mosaic_stage_eval": (_i32, [_vp, C.c_uint32, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "mosaic_planner_solve": (_i32, [_vp, _i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_double), _vp]),
    "mosaic_pool_reserve": (_i32, [_i32, _i32, _i32]),
    "mosaic_pool_get": (_i32, [_i32, _i32, _i32, C.POINTER(_vp)]),
    "mosaic_pool_creations": (_i64, []),
    "mosaic_pool_clear": (_i32, []),
    "mosaic_probe_placement": (_i32, [_vp, _i32, _vp]),
    "mosaic_module_create": (_i32, [C.POINTER(ModuleDesc), C.POINTER(_vp)]),
    "mosaic_module_destroy": (_i32, [_vp]),
    "mosaic_module_param_bytes": (_sz, [_vp]),
    "mosaic_module_workspace_bytes": (_sz, [_vp]),
    "mosaic_module_input_elems": (_sz, [_vp]),
    "mosaic_module_output_elems": (_sz, [_vp]),
    "mosaic_module_tensor_count": (_i32, [_vp]),
    "mosaic_module_tensor_info": (_i32, [_vp, _i32, C.c_char_p, C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64)]),
    "mosaic_module_bind": (_i32, [_vp, _vp, _vp, _vp, _sz]),
    "mosaic_module_bind_ids": (_i32, [_vp, _vp]),
    "mosaic_module_bind_image_counts": (_i32, [_vp, _vp]),
    "mosaic_module_forward": (_i32, [_vp, _i32, _vp, _vp, _vp]),
    "mosaic_module_backward": (_i32, [_vp, _i32, _vp, _vp, _vp]),
    "mosaic_module_step": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_module_optimizer_state_bytes": (C.c_size_t, [_vp, _i32]),
    "mosaic_module_adamw_step": (_i32, [_vp, _i32, _vp, _vp, C.c_size_t, _i32, _f32, _f32, _f32, _f32, _f32, _i64]),
    "mosaic_plan_validate": (_i32, [C.POINTER(Plan), _i32, _i32]),
    "mosaic_plan_stream_count": (_i32, [C.POINTER(Plan)]),
    "mosaic_device_hw_queues": (_i32, []),
    "mosaic_stage_run": (_i32, [C.POINTER(Stage), C.POINTER(Plan), C.POINTER(Timing)]),
    "mosaic_plan_choose": (_i32, [_i32, _i32, C.POINTER(_i32), C.POINTER(_f32), _i32, C.POINTER(_i32), C.POINTER(_f32)]),
    "mosaic_op_linear_fwd": (_i32, [_vp, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_linear_dgrad": (_i32, [_vp, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "mosaic_op_linear_wgrad": (_i32, [_vp, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_colsum_scratch_bytes": (_sz, [_i64]),
    "mosaic_op_linear_wgrad_scratch_bytes": (_sz, [_i64, _i64, _i64]),
    "mosaic_op_attention_fwd": (_i32, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]),
    "mosaic_op_attention_bwd": (_i32, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_attention_gqa_fwd": (_i32, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]),
    "mosaic_op_attention_gqa_bwd": (_i32, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_norm_fwd": (_i32, [_vp, _i32, _i32, _i32, _i64, _i64, _f32, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_norm_bwd_scratch_bytes": (_sz, [_i64]),
    "mosaic_op_norm_bwd": (_i32, [_vp, _i32, _i32, _i32, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_norm_bwd_static": (_i32, [_vp, _i32, _i32, _i32, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_norm_bwd_static_max_h": (_sz, []),
    "mosaic_op_gelu_fwd": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp]),
    "mosaic_op_gelu_bwd": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp, _vp]),
    "mosaic_op_gelu_tanh_fwd": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp]),
    "mosaic_op_gelu_tanh_bwd": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp, _vp]),
    "mosaic_op_rope_table_bytes": (C.c_size_t, [_i32, _i32]),
    "mosaic_op_rope_table": (_i32, [_vp, _i32, _i32, _i32, _f32, _vp]),
    "mosaic_op_rope": (_i32, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp]),
    "mosaic_op_adamw": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _f32, _f32, _i64]),
    "mosaic_op_swiglu_fwd": (_i32, [_vp, _i32, _i32, _i64, _i64, _vp, _vp]),
    "mosaic_op_swiglu_bwd": (_i32, [_vp, _i32, _i32, _i64, _i64, _vp, _vp, _vp]),
    "mosaic_op_linear_act_fwd": (_i32, [_vp, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_mse": (_i32, [_vp, _i32, _i32, _i64, _vp, _vp, _vp, _vp, _vp]),
    "mosaic_op_mse_scratch_bytes": (_sz, []),
}

_lib = None


def lib() -> C.CDLL:
    """Load libmosaic.so; raise if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_18710_amd.build` "
                               "or __graft_entry__.build(); there is no CPU fallback")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def check(status: int) -> None:
    if status != OK:
        raise MosaicError(status, lib().mosaic_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


# ------------------------------------------------------------------------------ device
def device_cu_count() -> int:
    n = lib().mosaic_device_cu_count()
    if n < 0:
        check(n)
    return n


def device_xcd_count() -> int:
    n = lib().mosaic_device_xcd_count()
    if n < 0:
        check(n)
    return n


def cu_mask_build(cu_total: int, n_xcd: int, quota: int, offset: int, layout: int) -> List[int]:
    nw = (cu_total + 31) // 32
    words = (C.c_uint32 * max(nw, 1))()
    check(lib().mosaic_cu_mask_build(cu_total, n_xcd, quota, offset, layout, words, nw))
    return [int(w) for w in words[:nw]]


class Stream:
    """A quota'd stream (owned by the library)."""

    def __init__(self, quota: int, offset: int = 0, layout: int = STRIPED, _handle=None, _pooled=False):
        if _handle is None:
            h = C.c_void_p()
            check(lib().mosaic_stream_create(quota, offset, layout, C.byref(h)))
            _handle = h.value
        self.handle = _handle
        self.pooled = _pooled

    @property
    def native(self) -> int:
        return lib().mosaic_stream_native(self.handle) or 0

    @property
    def quota(self) -> int:
        return lib().mosaic_stream_quota(self.handle)

    @property
    def offset(self) -> int:
        return lib().mosaic_stream_offset(self.handle)

    def destroy(self) -> None:
        if self.handle and not self.pooled:
            check(lib().mosaic_stream_destroy(self.handle))
        self.handle = None


def pool_reserve(quota: int, offset: int = 0, layout: int = STRIPED) -> None:
    check(lib().mosaic_pool_reserve(quota, offset, layout))


def pool_get(quota: int, offset: int = 0, layout: int = STRIPED) -> Stream:
    h = C.c_void_p()
    check(lib().mosaic_pool_get(quota, offset, layout, C.byref(h)))
    return Stream(quota, offset, layout, _handle=h.value, _pooled=True)


def pool_creations() -> int:
    return int(lib().mosaic_pool_creations())


def pool_clear() -> None:
    check(lib().mosaic_pool_clear())


def probe_placement(stream: Optional[Stream], n: int, out) -> None:
    check(lib().mosaic_probe_placement(stream.handle if stream else None, n, _ptr(out)))


# ----------------------------------------------------------------------------- modules
def make_desc(cfg: dict, dtype: str) -> ModuleDesc:
    d = ModuleDesc()
    d.kind = _KIND[cfg["kind"]]
    d.dtype = _DTYPE[dtype]
    for k in ("layers", "hidden", "heads", "mlp", "batch", "seq", "causal", "bias",
              "in_dim", "out_dim", "vocab", "n_img", "patch"):
        setattr(d, k, int(cfg.get(k, 0)))
    d.norm = _NORM[cfg.get("norm", "none")]
    d.act = _ACT[cfg.get("act", "gelu")]
    d.eps = float(cfg.get("eps", 0.0))
    d.rope_base = float(cfg.get("rope", 0.0) or 0.0)
    d.kv_heads = int(cfg.get("kv_heads", 0) or 0)
    return d


class Module:
    """One module m of a stage: descriptor + caller-owned device buffers."""

    def __init__(self, cfg: dict, dtype: str, device="cuda"):
        import torch
        self.cfg, self.dtype = dict(cfg), dtype
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        desc = make_desc(cfg, dtype)
        h = C.c_void_p()
        check(lib().mosaic_module_create(C.byref(desc), C.byref(h)))
        self.handle = h.value
        esize = 2 if dtype == "bf16" else 4
        self.param_elems = lib().mosaic_module_param_bytes(self.handle) // esize
        self.ws_bytes = lib().mosaic_module_workspace_bytes(self.handle)
        self.in_elems = lib().mosaic_module_input_elems(self.handle)
        self.out_elems = lib().mosaic_module_output_elems(self.handle)
        self.tensors: Dict[str, tuple] = {}
        name = C.create_string_buffer(32)
        off, rows, cols = C.c_int64(), C.c_int64(), C.c_int64()
        for i in range(lib().mosaic_module_tensor_count(self.handle)):
            check(lib().mosaic_module_tensor_info(self.handle, i, name, C.byref(off), C.byref(rows), C.byref(cols)))
            self.tensors[name.value.decode()] = (off.value, rows.value, cols.value)
        self.params = torch.zeros(max(self.param_elems, 8), dtype=self.tdtype, device=device)
        self.grads = torch.zeros(max(self.param_elems, 8), dtype=self.tdtype, device=device)
        self.workspace = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self._ws_ptr = ws_ptr
        check(lib().mosaic_module_bind(self.handle, self.params.data_ptr(), self.grads.data_ptr(),
                                       ws_ptr, self.ws_bytes))
        self._ids = None

    def set_tensor(self, name: str, value: np.ndarray) -> None:
        import torch
        off, rows, cols = self.tensors[name]
        v = torch.from_numpy(np.ascontiguousarray(value, dtype=np.float32).reshape(-1))
        assert v.numel() == rows * cols, (name, v.numel(), rows, cols)
        self.params[off:off + rows * cols].copy_(v.to(self.tdtype))

    def get_tensor(self, name: str, grads: bool = False) -> np.ndarray:
        off, rows, cols = self.tensors[name]
        src = self.grads if grads else self.params
        return src[off:off + rows * cols].float().cpu().numpy().reshape(rows, cols).astype(np.float64)

    def bind_ids(self, ids) -> None:
        self._ids = ids
        check(lib().mosaic_module_bind_ids(self.handle, ids.data_ptr()))

    def bind_image_counts(self, counts) -> None:
        self._counts = counts
        check(lib().mosaic_module_bind_image_counts(self.handle, _ptr(counts)))

    def forward(self, quota: int, stream: Optional[Stream], x, y) -> None:
        check(lib().mosaic_module_forward(self.handle, quota, stream.handle if stream else None, _ptr(x), _ptr(y)))

    def backward(self, quota: int, stream: Optional[Stream], dy, dx=None) -> None:
        check(lib().mosaic_module_backward(self.handle, quota, stream.handle if stream else None, _ptr(dy), _ptr(dx)))

    def step(self, quota: int, stream: Optional[Stream], x, y, dy=None, target=None, dx=None, loss=None) -> None:
        check(lib().mosaic_module_step(self.handle, quota, stream.handle if stream else None, _ptr(x), _ptr(dy),
                                       _ptr(target), _ptr(y), _ptr(dx), _ptr(loss)))

    def init_optimizer(self, use_master: bool = False) -> None:
        """Allocates the AdamW state (zero moments; the master copy, if asked for, starts as
        the current parameters)."""
        import torch
        n = lib().mosaic_module_optimizer_state_bytes(self.handle, int(use_master)) // 4
        self.opt_state = torch.zeros(n, dtype=torch.float32, device=self.params.device)
        self.use_master = bool(use_master)
        if use_master:
            self.opt_state[2 * self.param_elems:3 * self.param_elems].copy_(self.params[:self.param_elems].float())

    def adamw_step(self, quota: int, stream: Optional[Stream], step: int, lr: float, beta1: float = 0.9,
                   beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.0) -> None:
        check(lib().mosaic_module_adamw_step(self.handle, quota, stream.handle if stream else None, _ptr(self.opt_state),
                                             self.opt_state.numel() * 4, int(self.use_master), lr, beta1, beta2, eps,
                                             weight_decay, step))

    def destroy(self) -> None:
        if self.handle:
            lib().mosaic_module_destroy(self.handle)
            self.handle = None


# ------------------------------------------------------------------------------ stages
def _vp_array(items: Sequence) -> "C.Array":
    arr = (C.c_void_p * len(items))()
    for i, it in enumerate(items):
        arr[i] = _ptr(it)
    return arr


def make_plan(quotas: Sequence[int], offsets: Sequence[int], layout: int, mode: int):
    n = len(quotas)
    q = (C.c_int32 * n)(*quotas)
    o = (C.c_int32 * n)(*offsets)
    p = Plan(n, q, o, layout, mode)
    p._keep = (q, o)
    return p


def plan_validate(quotas, offsets, layout, mode, cu_total: int, n_xcd: int) -> None:
    p = make_plan(quotas, offsets, layout, mode)
    check(lib().mosaic_plan_validate(C.byref(p), cu_total, n_xcd))


def plan_stream_count(quotas, offsets, layout, mode) -> int:
    p = make_plan(quotas, offsets, layout, mode)
    return int(lib().mosaic_plan_stream_count(C.byref(p)))


def device_hw_queues() -> int:
    return int(lib().mosaic_device_hw_queues())


def stage_run(modules: Sequence[Module], x, y, quotas, offsets, layout=STRIPED, mode=COLOCATED,
              dy=None, target=None, dx=None, loss=None) -> dict:
    n = len(modules)
    none = [None] * n
    st = Stage()
    st.n = n
    handles = (C.c_void_p * n)(*[m.handle for m in modules])
    arrays = [handles, _vp_array(x), _vp_array(dy or none), _vp_array(target or none), _vp_array(y),
              _vp_array(dx or none), _vp_array(loss or none)]
    st.modules, st.x, st.dy, st.target, st.y, st.dx, st.loss = arrays
    p = make_plan(quotas, offsets, layout, mode)
    t = Timing()
    check(lib().mosaic_stage_run(C.byref(st), C.byref(p), C.byref(t)))
    return dict(stage_ms=float(t.stage_ms), module_ms=[float(t.module_ms[i]) for i in range(n)])


def plan_choose(cu_points: Sequence[int], times: Sequence[Sequence[float]], cu_total: int):
    n_mod, n_pts = len(times), len(cu_points)
    pts = (C.c_int32 * n_pts)(*cu_points)
    flat = (C.c_float * (n_mod * n_pts))(*[float(v) for row in times for v in row])
    out = (C.c_int32 * n_mod)()
    tout = C.c_float()
    check(lib().mosaic_plan_choose(n_mod, n_pts, pts, flat, cu_total, out, C.byref(tout)))
    return [int(v) for v in out], float(tout.value)


# ------------------------------------------------- performance-model correction, planner
ADDITIVE, COMPOSITE = 0, 1
EARLY_PRUNE, CACHE = 1, 2
DELAY_ABSOLUTE, DELAY_PEER_RELATIVE = 0, 1


def interference_delta(e: Sequence[float], bw: Sequence[float]) -> float:
    ev = (C.c_double * 3)(*[float(v) for v in e])
    b = (C.c_double * max(1, len(bw)))(*[float(v) for v in bw])
    return float(lib().mosaic_interference_delta(ev, len(bw), b))


def interference_fit(groups: Sequence[Sequence[float]], delta: Sequence[float], model: int = COMPOSITE):
    n = len(groups)
    sizes = (C.c_int32 * max(1, n))(*[len(g) for g in groups])
    flat = [float(v) for g in groups for v in g]
    bw = (C.c_double * max(1, len(flat)))(*flat)
    d = (C.c_double * max(1, n))(*[float(v) for v in delta])
    e = (C.c_double * 3)()
    r2 = C.c_double()
    check(lib().mosaic_interference_fit(n, sizes, bw, d, model, e, C.byref(r2)))
    return [float(v) for v in e], float(r2.value)


class _PlannerProblem(C.Structure):
    _fields_ = [("n_modules", C.c_int32), ("n_edges", C.c_int32), ("edges", C.POINTER(C.c_int32)),
                ("n_points", C.c_int32), ("cu_points", C.POINTER(C.c_int32)), ("times", C.POINTER(C.c_double)),
                ("bw", C.POINTER(C.c_double)), ("e", C.POINTER(C.c_double)), ("cu_total", C.c_int32),
                ("delay_form", C.c_int32)]


class _PlannerStats(C.Structure):
    _fields_ = [("stage_evals", C.c_int64), ("cache_hits", C.c_int64), ("pruned", C.c_int64), ("rounds", C.c_int64)]


def _planner_problem(n_modules, edges, cu_points, times, cu_total, bw=None, e=None, form=0):
    keep = []          # ctypes arrays the struct points into
    def arr(ty, vals):
        a = (ty * max(1, len(vals)))(*vals)
        keep.append(a)
        return a
    p = _PlannerProblem()
    p.n_modules, p.n_edges, p.n_points, p.cu_total = n_modules, len(edges), len(cu_points), cu_total
    p.delay_form = form
    p.edges = arr(C.c_int32, [int(v) for ed in edges for v in ed])
    p.cu_points = arr(C.c_int32, [int(v) for v in cu_points])
    p.times = arr(C.c_double, [float(v) for row in times for v in row])
    if bw is not None:
        p.bw = arr(C.c_double, [float(v) for row in bw for v in row])
        p.e = arr(C.c_double, [float(v) for v in e])
    return p, keep


def stage_eval(modules: Sequence[int], n_modules: int, cu_points, times, cu_total: int, bw=None, e=None, form: int = 0):
    """StageEval for the stage holding `modules`: (time in ms, {module: CUs})."""
    p, keep = _planner_problem(n_modules, [], cu_points, times, cu_total, bw, e, form)
    mask = 0
    for m in modules:
        mask |= 1 << m
    q = (C.c_int32 * n_modules)()
    t = C.c_double()
    check(lib().mosaic_stage_eval(C.byref(p), mask, q, C.byref(t)))
    return float(t.value), {m: int(q[m]) for m in modules if q[m] > 0}


def planner_solve(n_modules: int, edges, cu_points, times, cu_total: int, bw=None, e=None, flags: int = EARLY_PRUNE | CACHE,
                  form: int = 0):
    """Alg. 1: (stages in execution order as lists of modules, {module: CUs}, iteration time, stats)."""
    p, keep = _planner_problem(n_modules, edges, cu_points, times, cu_total, bw, e, form)
    so, qo = (C.c_int32 * n_modules)(), (C.c_int32 * n_modules)()
    ns, t, st = C.c_int32(), C.c_double(), _PlannerStats()
    check(lib().mosaic_planner_solve(C.byref(p), flags, so, qo, C.byref(ns), C.byref(t), C.byref(st)))
    stages = [[m for m in range(n_modules) if so[m] == i] for i in range(ns.value)]
    stats = dict(stage_evals=int(st.stage_evals), cache_hits=int(st.cache_hits), pruned=int(st.pruned), rounds=int(st.rounds))
    return stages, {m: int(qo[m]) for m in range(n_modules)}, float(t.value), stats


# ------------------------------------------------------------------- single operations
def _dt(dtype: str) -> int:
    return _DTYPE[dtype]


def op_linear_fwd(stream, quota, dtype, T, k, n, X, W, bias, R, Y):
    check(lib().mosaic_op_linear_fwd(stream, quota, _dt(dtype), T, k, n, _ptr(X), _ptr(W), _ptr(bias), _ptr(R), _ptr(Y)))


def op_linear_dgrad(stream, quota, dtype, T, k, n, dY, W, R, dX):
    check(lib().mosaic_op_linear_dgrad(stream, quota, _dt(dtype), T, k, n, _ptr(dY), _ptr(W), _ptr(R), _ptr(dX)))


def op_linear_wgrad(stream, quota, dtype, T, k, n, X, dY, dW, db, scratch):
    check(lib().mosaic_op_linear_wgrad(stream, quota, _dt(dtype), T, k, n, _ptr(X), _ptr(dY), _ptr(dW), _ptr(db), _ptr(scratch)))


def op_attention_fwd(stream, quota, dtype, B, N, H, d, causal, qkv, O, lse):
    check(lib().mosaic_op_attention_fwd(stream, quota, _dt(dtype), B, N, H, d, causal, _ptr(qkv), _ptr(O), _ptr(lse)))


def op_attention_bwd(stream, quota, dtype, B, N, H, d, causal, qkv, O, lse, dO, dqkv, delta):
    check(lib().mosaic_op_attention_bwd(stream, quota, _dt(dtype), B, N, H, d, causal, _ptr(qkv), _ptr(O), _ptr(lse),
                                        _ptr(dO), _ptr(dqkv), _ptr(delta)))


def op_attention_gqa_fwd(stream, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse):
    check(lib().mosaic_op_attention_gqa_fwd(stream, quota, _dt(dtype), B, N, H, Hkv, d, causal, _ptr(qkv), _ptr(O), _ptr(lse)))


def op_attention_gqa_bwd(stream, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse, dO, dqkv, delta):
    check(lib().mosaic_op_attention_gqa_bwd(stream, quota, _dt(dtype), B, N, H, Hkv, d, causal, _ptr(qkv), _ptr(O), _ptr(lse),
                                            _ptr(dO), _ptr(dqkv), _ptr(delta)))


def op_norm_fwd(stream, quota, dtype, norm, T, h, eps, x, gamma, beta, y, stats):
    check(lib().mosaic_op_norm_fwd(stream, quota, _dt(dtype), _NORM[norm], T, h, eps, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(stats)))


def op_norm_bwd(stream, quota, dtype, norm, T, h, x, gamma, stats, dy, R, dx, dgamma, dbeta, scratch):
    check(lib().mosaic_op_norm_bwd(stream, quota, _dt(dtype), _NORM[norm], T, h, _ptr(x), _ptr(gamma), _ptr(stats), _ptr(dy),
                                   _ptr(R), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(scratch)))


def op_norm_bwd_static(stream, quota, dtype, norm, T, h, x, gamma, stats, dy, R, dx, dgamma, dbeta):
    check(lib().mosaic_op_norm_bwd_static(stream, quota, _dt(dtype), _NORM[norm], T, h, _ptr(x), _ptr(gamma), _ptr(stats),
                                          _ptr(dy), _ptr(R), _ptr(dx), _ptr(dgamma), _ptr(dbeta)))


def norm_bwd_static_max_h() -> int:
    return int(lib().mosaic_op_norm_bwd_static_max_h())


def op_gelu_fwd(stream, quota, dtype, n, z, a):
    check(lib().mosaic_op_gelu_fwd(stream, quota, _dt(dtype), n, _ptr(z), _ptr(a)))


def op_gelu_bwd(stream, quota, dtype, n, z, da, dz):
    check(lib().mosaic_op_gelu_bwd(stream, quota, _dt(dtype), n, _ptr(z), _ptr(da), _ptr(dz)))


def op_gelu_tanh_fwd(stream, quota, dtype, n, z, a):
    check(lib().mosaic_op_gelu_tanh_fwd(stream, quota, _dt(dtype), n, _ptr(z), _ptr(a)))


def op_gelu_tanh_bwd(stream, quota, dtype, n, z, da, dz):
    check(lib().mosaic_op_gelu_tanh_bwd(stream, quota, _dt(dtype), n, _ptr(z), _ptr(da), _ptr(dz)))


def rope_table_bytes(N, d) -> int:
    return int(lib().mosaic_op_rope_table_bytes(N, d))


def op_rope_table(stream, quota, N, d, base, table):
    check(lib().mosaic_op_rope_table(stream, quota, N, d, base, _ptr(table)))


def op_rope(stream, quota, dtype, B, N, H, d, direction, qkv, table):
    check(lib().mosaic_op_rope(stream, quota, _dt(dtype), B, N, H, d, direction, _ptr(qkv), _ptr(table)))


def op_adamw(stream, quota, dtype, n, params, grads, m, v, master, lr, beta1, beta2, eps, weight_decay, step):
    check(lib().mosaic_op_adamw(stream, quota, _dt(dtype), n, _ptr(params), _ptr(grads), _ptr(m), _ptr(v), _ptr(master),
                                lr, beta1, beta2, eps, weight_decay, step))


def op_swiglu_fwd(stream, quota, dtype, T, f, gu, a):
    check(lib().mosaic_op_swiglu_fwd(stream, quota, _dt(dtype), T, f, _ptr(gu), _ptr(a)))


def op_linear_act_fwd(stream, quota, dtype, act, T, k, n, X, W, bias, Z, A):
    check(lib().mosaic_op_linear_act_fwd(stream, quota, _dt(dtype), act, T, k, n, _ptr(X), _ptr(W), _ptr(bias), _ptr(Z), _ptr(A)))


def op_swiglu_bwd(stream, quota, dtype, T, f, gu, da, dgu):
    check(lib().mosaic_op_swiglu_bwd(stream, quota, _dt(dtype), T, f, _ptr(gu), _ptr(da), _ptr(dgu)))


def op_mse(stream, quota, dtype, n, y, target, dy, loss, scratch):
    check(lib().mosaic_op_mse(stream, quota, _dt(dtype), n, _ptr(y), _ptr(target), _ptr(dy), _ptr(loss), _ptr(scratch)))


def norm_bwd_scratch_bytes(h: int) -> int:
    return int(lib().mosaic_op_norm_bwd_scratch_bytes(h))


def colsum_scratch_bytes(n: int) -> int:
    return int(lib().mosaic_op_colsum_scratch_bytes(n))


def linear_wgrad_scratch_bytes(T: int, k: int, n: int) -> int:
    return int(lib().mosaic_op_linear_wgrad_scratch_bytes(T, k, n))


def mse_scratch_bytes() -> int:
    return int(lib().mosaic_op_mse_scratch_bytes())
