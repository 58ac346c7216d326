"""ctypes binding of libvorta.so: one Python function per C entry point, same names.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
torch is used for device memory and streams; routes and gates are host arrays.
"""
import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvorta.so")

VORTA_F32, VORTA_BF16 = 0, 1
VORTA_LAYOUT_NHD, VORTA_LAYOUT_HND = 0, 1
VORTA_CENTER_CLAMP, VORTA_CENTER_IDENTITY = 0, 1
VORTA_MAX_HEADS = 128

SYMBOLS = [
    "vorta_strerror", "vorta_last_error", "vorta_plan_create", "vorta_plan_destroy", "vorta_plan_info_get",
    "vorta_tile_permutation", "vorta_tile_row0", "vorta_window_boxes", "vorta_window_runs", "vorta_bcs_slot_bases",
    "vorta_probe_mfma_rate", "vorta_route_partition", "vorta_router_gates", "vorta_route_select", "vorta_reorder_to_tiles", "vorta_reorder_from_tiles",
    "vorta_bcs_build_index", "vorta_bcs_pool", "vorta_attention_routed", "vorta_scatter_back",
    "vorta_workspace_bytes", "vorta_workspace_layout", "vorta_routed_attention_layer",
    "vorta_soft_mixture_workspace_bytes", "vorta_soft_mixture_layer",
]


class VortaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"vorta error {code}: {message}")
        self.code = code


class vorta_layer_desc(ctypes.Structure):
    _fields_ = [
        ("F", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
        ("n_text", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("layout", ctypes.c_int32),
        ("tile", ctypes.c_int32 * 3), ("window", ctypes.c_int32 * 3), ("center_mode", ctypes.c_int32),
        ("bucket", ctypes.c_int32 * 3), ("keep_num", ctypes.c_int32), ("keep_den", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
    ]


class vorta_plan_info(ctypes.Structure):
    _fields_ = [
        ("n_video", ctypes.c_int64), ("n_tokens", ctypes.c_int64), ("tiles", ctypes.c_int32 * 3),
        ("n_tiles", ctypes.c_int32), ("tile_tokens", ctypes.c_int32), ("window_key_tiles", ctypes.c_int32),
        ("max_runs", ctypes.c_int32), ("n_buckets", ctypes.c_int32), ("n_core", ctypes.c_int64),
        ("n_core_tokens", ctypes.c_int64), ("elem_bytes", ctypes.c_int32),
    ]


class vorta_attn_io(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("q", "k", "v", "out", "q_t", "k_t", "v_t", "o_t", "q_c", "k_c", "v_c", "o_c")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the in-tree libvorta.so, building it first if it is not there.
    There is no fallback: without the library nothing in this package computes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    lib.vorta_strerror.restype = ctypes.c_char_p
    lib.vorta_strerror.argtypes = [ctypes.c_int]
    lib.vorta_last_error.restype = ctypes.c_char_p
    for name in SYMBOLS[2:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        lib = load_library()
        msg = lib.vorta_last_error().decode() or lib.vorta_strerror(rc).decode()
        raise VortaError(rc, msg)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise VortaError(-1, "device tensor expected (the library has no CPU path)")
    if not t.is_contiguous():
        raise VortaError(-1, "contiguous tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _routes(routes) -> np.ndarray:
    if isinstance(routes, torch.Tensor):
        routes = routes.cpu().numpy()
    return np.ascontiguousarray(np.asarray(routes, dtype=np.uint8))


def _u8p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


class Plan:
    """Owner of a vorta_plan*; info fields are attributes."""

    def __init__(self, handle, desc: vorta_layer_desc):
        self.handle = handle
        self.desc = desc
        info = vorta_plan_info()
        _check(load_library().vorta_plan_info_get(handle, ctypes.byref(info)))
        self.n_video, self.n_tokens = info.n_video, info.n_tokens
        self.tiles = tuple(info.tiles)
        self.n_tiles, self.tile_tokens = info.n_tiles, info.tile_tokens
        self.window_key_tiles, self.max_runs = info.window_key_tiles, info.max_runs
        self.n_buckets, self.n_core, self.n_core_tokens = info.n_buckets, info.n_core, info.n_core_tokens
        self.elem_bytes = info.elem_bytes
        self.heads, self.head_dim = desc.heads, desc.head_dim
        self.torch_dtype = torch.bfloat16 if desc.dtype == VORTA_BF16 else torch.float32

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.vorta_plan_destroy(self.handle)
            self.handle = None


def vorta_plan_create(grid, heads, head_dim, dtype, tile, window, *, n_text=0, layout=VORTA_LAYOUT_HND,
                      center_mode=VORTA_CENTER_CLAMP, bucket=(2, 3, 2), keep_num=1, keep_den=2,
                      softmax_scale=0.0) -> Plan:
    lib = load_library()
    if isinstance(dtype, str):
        dtype = {"fp32": VORTA_F32, "bf16": VORTA_BF16}[dtype]
    d = vorta_layer_desc(grid[0], grid[1], grid[2], n_text, heads, head_dim, dtype, layout,
                         (ctypes.c_int32 * 3)(*tile), (ctypes.c_int32 * 3)(*window), center_mode,
                         (ctypes.c_int32 * 3)(*bucket), keep_num, keep_den, softmax_scale)
    handle = ctypes.c_void_p()
    _check(lib.vorta_plan_create(ctypes.byref(d), ctypes.byref(handle)))
    return Plan(handle, d)


def plan_for(cfg, layout=VORTA_LAYOUT_HND, **over) -> Plan:
    """Plan for a synth_inputs.LayerConfig-like object (attribute access only)."""
    kw = dict(grid=cfg.grid, heads=cfg.heads, head_dim=cfg.head_dim, dtype=cfg.dtype, tile=cfg.tile,
              window=cfg.window, n_text=cfg.n_text, layout=layout, bucket=cfg.bucket,
              keep_num=cfg.keep_num, keep_den=cfg.keep_den)
    kw.update(over)
    return vorta_plan_create(**kw)


def vorta_plan_destroy(plan: Plan):
    if plan.handle:
        _check(load_library().vorta_plan_destroy(plan.handle))
        plan.handle = None


# ---- host tables ---------------------------------------------------------------------------

def vorta_tile_permutation(plan: Plan) -> np.ndarray:
    perm = np.empty(plan.n_video, dtype=np.int32)
    _check(load_library().vorta_tile_permutation(plan.handle, _i32p(perm)))
    return perm


def vorta_tile_row0(plan: Plan) -> np.ndarray:
    row0 = np.empty(plan.n_tiles + 1, dtype=np.int32)
    _check(load_library().vorta_tile_row0(plan.handle, _i32p(row0)))
    return row0


def vorta_window_boxes(plan: Plan) -> np.ndarray:
    boxes = np.empty((plan.n_tiles, 6), dtype=np.int32)
    _check(load_library().vorta_window_boxes(plan.handle, _i32p(boxes)))
    return boxes


def vorta_window_runs(plan: Plan):
    runs = np.empty((plan.n_tiles, plan.max_runs, 2), dtype=np.int32)
    n_runs = np.empty(plan.n_tiles, dtype=np.int32)
    _check(load_library().vorta_window_runs(plan.handle, _i32p(runs), _i32p(n_runs)))
    return runs, n_runs


def vorta_bcs_slot_bases(plan: Plan) -> np.ndarray:
    sb = np.empty(plan.n_buckets + 1, dtype=np.int32)
    _check(load_library().vorta_bcs_slot_bases(plan.handle, _i32p(sb)))
    return sb


def vorta_route_partition(plan: Plan, routes):
    r = _routes(routes)
    heads = np.empty(plan.heads, dtype=np.int32)
    counts = np.empty(3, dtype=np.int32)
    _check(load_library().vorta_route_partition(plan.handle, _u8p(r), _i32p(heads), _i32p(counts)))
    return heads, counts


def vorta_router_gates(t_emb, w_r) -> np.ndarray:
    t = np.ascontiguousarray(t_emb, dtype=np.float32)
    w = np.ascontiguousarray(w_r, dtype=np.float32)
    heads, d_t = w.shape[0], t.shape[0]
    assert w.shape == (heads, d_t, 3)
    alpha = np.empty((heads, 3), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    _check(load_library().vorta_router_gates(t.ctypes.data_as(fp), w.ctypes.data_as(fp), d_t, heads,
                                             alpha.ctypes.data_as(fp)))
    return alpha


def vorta_probe_mfma_rate(operands: torch.Tensor, iters: int, workgroups: int, stream=None):
    """Returns (FLOPs issued, sink, clocks); the caller times the call with events."""
    assert operands.numel() * operands.element_size() >= 16 * 64 * 16
    sink = torch.empty(workgroups * 512, dtype=torch.float32, device=operands.device)
    clocks = torch.zeros(2, dtype=torch.int64, device=operands.device)
    _check(load_library().vorta_probe_mfma_rate(_ptr(operands), iters, workgroups, _ptr(sink), _ptr(clocks),
                                                _stream(stream)))
    return workgroups * 8 * iters * 32 * 32768.0, sink, clocks


def vorta_route_select(alpha) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    routes = np.empty(a.shape[0], dtype=np.uint8)
    _check(load_library().vorta_route_select(a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                             ctypes.c_int32(a.shape[0]), _u8p(routes)))
    return routes


# ---- device passes -------------------------------------------------------------------------

def _count(routes: np.ndarray, r: int) -> int:
    return int((routes == r).sum())


def vorta_reorder_to_tiles(plan: Plan, src: torch.Tensor, routes, dst: torch.Tensor = None, stream=None):
    r = _routes(routes)
    if dst is None:
        dst = torch.empty(_count(r, 1), plan.n_tokens, plan.head_dim, dtype=src.dtype, device=src.device)
    _check(load_library().vorta_reorder_to_tiles(plan.handle, _ptr(src), _u8p(r), _ptr(dst), _stream(stream)))
    return dst


def vorta_reorder_from_tiles(plan: Plan, src: torch.Tensor, routes, dst: torch.Tensor, stream=None):
    r = _routes(routes)
    _check(load_library().vorta_reorder_from_tiles(plan.handle, _ptr(src), _u8p(r), _ptr(dst), _stream(stream)))
    return dst


def vorta_bcs_build_index(plan: Plan, feat: torch.Tensor, routes, keep_idx=None, assign=None, stream=None):
    r = _routes(routes)
    n = _count(r, 2)
    if keep_idx is None:
        keep_idx = torch.empty(n, plan.n_core, dtype=torch.int32, device=feat.device)
    if assign is None:
        assign = torch.empty(n, plan.n_video, dtype=torch.int32, device=feat.device)
    _check(load_library().vorta_bcs_build_index(plan.handle, _ptr(feat), _u8p(r), _ptr(keep_idx), _ptr(assign),
                                                _stream(stream)))
    return keep_idx, assign


def vorta_bcs_pool(plan: Plan, src: torch.Tensor, routes, keep_idx, assign, dst=None, stream=None):
    r = _routes(routes)
    if dst is None:
        dst = torch.empty(_count(r, 2), plan.n_core_tokens, plan.head_dim, dtype=src.dtype, device=src.device)
    _check(load_library().vorta_bcs_pool(plan.handle, _ptr(src), _u8p(r), _ptr(keep_idx), _ptr(assign),
                                         _ptr(dst), _stream(stream)))
    return dst


def vorta_attention_routed(plan: Plan, routes, *, q=None, k=None, v=None, out=None, q_t=None, k_t=None,
                           v_t=None, o_t=None, q_c=None, k_c=None, v_c=None, o_c=None, stream=None):
    r = _routes(routes)
    io = vorta_attn_io(*[_ptr(t).value for t in (q, k, v, out, q_t, k_t, v_t, o_t, q_c, k_c, v_c, o_c)])
    _check(load_library().vorta_attention_routed(plan.handle, _u8p(r), ctypes.byref(io), _stream(stream)))


def vorta_scatter_back(plan: Plan, routes, o_t, o_c, assign, out: torch.Tensor, stream=None):
    r = _routes(routes)
    _check(load_library().vorta_scatter_back(plan.handle, _u8p(r), _ptr(o_t), _ptr(o_c), _ptr(assign), _ptr(out),
                                             _stream(stream)))
    return out


def vorta_workspace_bytes(plan: Plan, routes) -> int:
    r = _routes(routes)
    n = ctypes.c_size_t()
    _check(load_library().vorta_workspace_bytes(plan.handle, _u8p(r), ctypes.byref(n)))
    return n.value


def vorta_workspace_layout(plan: Plan, routes) -> Sequence[int]:
    r = _routes(routes)
    off = (ctypes.c_size_t * 10)()
    _check(load_library().vorta_workspace_layout(plan.handle, _u8p(r), off))
    return list(off)


def vorta_routed_attention_layer(plan: Plan, q, k, v, routes, out=None, workspace=None, stream=None):
    r = _routes(routes)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(vorta_workspace_bytes(plan, r), dtype=torch.uint8, device=q.device)
    _check(load_library().vorta_routed_attention_layer(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), _u8p(r), _ptr(out), _ptr(workspace),
        ctypes.c_size_t(workspace.numel()), _stream(stream)))
    return out


def vorta_soft_mixture_workspace_bytes(plan: Plan) -> int:
    n = ctypes.c_size_t()
    _check(load_library().vorta_soft_mixture_workspace_bytes(plan.handle, ctypes.byref(n)))
    return n.value


def vorta_soft_mixture_layer(plan: Plan, q, k, v, alpha, out=None, workspace=None, stream=None):
    a = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(vorta_soft_mixture_workspace_bytes(plan), dtype=torch.uint8, device=q.device)
    _check(load_library().vorta_soft_mixture_layer(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _ptr(out),
        _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(stream)))
    return out
