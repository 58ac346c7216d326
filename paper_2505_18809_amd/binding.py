"""ctypes binding of libvorta.so: one Python function per C entry point, same names.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
torch is used for device memory and streams; routes and gates are host arrays.

The C ABI takes raw pointers, so this layer is where tensor arguments can still be checked
against the plan: dtype, exact shape for the plan's layout, contiguity, one common device,
route and gate array lengths.  A mismatch raises VortaError before anything is launched (inside
a kernel it would be an out-of-bounds device access).
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
VORTA_CENTER_CLAMP, VORTA_CENTER_IDENTITY, VORTA_CENTER_BLOCK = 0, 1, 2
VORTA_MAX_HEADS = 128
VORTA_FEAT_USER_LAYOUT = -1
VORTA_STATIC_SCRATCH_BYTES = 32 << 20

SYMBOLS = [
    "vorta_strerror", "vorta_last_error", "vorta_plan_create", "vorta_plan_destroy", "vorta_plan_info_get",
    "vorta_tile_permutation", "vorta_tile_row0", "vorta_window_boxes", "vorta_window_runs", "vorta_window_items",
    "vorta_bcs_slot_bases",
    "vorta_plan_upload", "vorta_route_partition", "vorta_router_gates", "vorta_route_select", "vorta_router_device",
    "vorta_reorder_to_tiles", "vorta_reorder_from_tiles",
    "vorta_bcs_build_index", "vorta_bcs_pool", "vorta_bcs_select_pool", "vorta_rope_apply", "vorta_attention_routed", "vorta_scatter_back",
    "vorta_workspace_bytes", "vorta_workspace_layout", "vorta_routed_attention_layer",
    "vorta_soft_mixture_workspace_bytes", "vorta_soft_mixture_layer", "vorta_routed_attention_layer_static",
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
        ("rope_dims", ctypes.c_int32 * 3), ("rope_theta", ctypes.c_float),
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


def _routes(routes, plan: "Plan" = None) -> np.ndarray:
    if isinstance(routes, torch.Tensor):
        routes = routes.cpu().numpy()
    r = np.ascontiguousarray(np.asarray(routes, dtype=np.uint8)).reshape(-1)
    if plan is not None and r.shape[0] != plan.heads:
        raise VortaError(-1, f"routes has {r.shape[0]} entries, the plan has {plan.heads} heads")
    return r


def _check_tensors(plan: "Plan", **named):
    """named: name -> (tensor or None, expected shape, expected dtype).  Every given tensor must
    be a contiguous device tensor of exactly that shape and dtype, all on one device."""
    device = None
    for name, (t, shape, dtype) in named.items():
        if t is None:
            continue
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise VortaError(-1, f"{name}: device tensor expected (the library has no CPU path)")
        if t.dtype != dtype:
            raise VortaError(-3, f"{name}: dtype {t.dtype}, the plan needs {dtype}")
        if tuple(t.shape) != tuple(shape):
            raise VortaError(-2, f"{name}: shape {tuple(t.shape)}, the plan needs {tuple(shape)}")
        if not t.is_contiguous():
            raise VortaError(-1, f"{name}: contiguous tensor expected")
        if device is None:
            device = t.device
        elif t.device != device:
            raise VortaError(-1, f"{name} is on {t.device}, other arguments on {device}")


def _check_workspace(ws):
    if ws is None:
        return
    if not isinstance(ws, torch.Tensor) or not ws.is_cuda or ws.dtype != torch.uint8 or ws.dim() != 1 \
            or not ws.is_contiguous():
        raise VortaError(-1, "workspace: a contiguous 1-D uint8 device tensor expected")


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
        self.layout = desc.layout

    def user_shape(self):
        """Shape of q, k, v, out in the plan's layout."""
        if self.layout == VORTA_LAYOUT_NHD:
            return (self.n_tokens, self.heads, self.head_dim)
        return (self.heads, self.n_tokens, self.head_dim)

    def _user(self, t):
        return (t, self.user_shape(), self.torch_dtype)

    def _tiled(self, t, n):
        return (t, (n, self.n_tokens, self.head_dim), self.torch_dtype)

    def _core(self, t, n):
        return (t, (n, self.n_core_tokens, self.head_dim), self.torch_dtype)

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.vorta_plan_destroy(self.handle)
            self.handle = None


def vorta_plan_create(grid, heads, head_dim, dtype, tile, window, *, n_text=0, layout=VORTA_LAYOUT_HND,
                      center_mode=VORTA_CENTER_CLAMP, bucket=(2, 3, 2), keep_num=1, keep_den=2,
                      softmax_scale=0.0, rope_dims=(0, 0, 0), rope_theta=0.0) -> Plan:
    lib = load_library()
    if isinstance(dtype, str):
        dtype = {"fp32": VORTA_F32, "bf16": VORTA_BF16}[dtype]
    d = vorta_layer_desc(grid[0], grid[1], grid[2], n_text, heads, head_dim, dtype, layout,
                         (ctypes.c_int32 * 3)(*tile), (ctypes.c_int32 * 3)(*window), center_mode,
                         (ctypes.c_int32 * 3)(*bucket), keep_num, keep_den, softmax_scale,
                         (ctypes.c_int32 * 3)(*(rope_dims or (0, 0, 0))), rope_theta)
    handle = ctypes.c_void_p()
    _check(lib.vorta_plan_create(ctypes.byref(d), ctypes.byref(handle)))
    return Plan(handle, d)


def plan_for(cfg, layout=VORTA_LAYOUT_HND, **over) -> Plan:
    """Plan for a synth_inputs.LayerConfig-like object (attribute access only)."""
    kw = dict(grid=cfg.grid, heads=cfg.heads, head_dim=cfg.head_dim, dtype=cfg.dtype, tile=cfg.tile,
              window=cfg.window, n_text=cfg.n_text, layout=layout, bucket=cfg.bucket,
              keep_num=cfg.keep_num, keep_den=cfg.keep_den,
              rope_dims=getattr(cfg, "rope_dims", None) or (0, 0, 0), rope_theta=getattr(cfg, "rope_theta", 0.0))
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


def vorta_window_items(plan: Plan):
    """(items of more than 128 rows, items of at most 128 rows), each int32 [n, 4] = tile, tile, tile, count."""
    counts = np.zeros(2, dtype=np.int32)
    _check(load_library().vorta_window_items(plan.handle, None, _i32p(counts)))
    items = np.zeros((int(counts.sum()), 4), dtype=np.int32)
    if len(items):
        _check(load_library().vorta_window_items(plan.handle, _i32p(items), _i32p(counts)))
    return items[:counts[0]], items[counts[0]:]


def vorta_bcs_slot_bases(plan: Plan) -> np.ndarray:
    sb = np.empty(plan.n_buckets + 1, dtype=np.int32)
    _check(load_library().vorta_bcs_slot_bases(plan.handle, _i32p(sb)))
    return sb


def vorta_route_partition(plan: Plan, routes):
    r = _routes(routes, plan)
    heads = np.empty(plan.heads, dtype=np.int32)
    counts = np.empty(3, dtype=np.int32)
    _check(load_library().vorta_route_partition(plan.handle, _u8p(r), _i32p(heads), _i32p(counts)))
    return heads, counts


def vorta_router_gates(t_emb, w_r) -> np.ndarray:
    t = np.ascontiguousarray(t_emb, dtype=np.float32)
    w = np.ascontiguousarray(w_r, dtype=np.float32)
    if t.ndim != 1 or w.ndim != 3 or w.shape[1:] != (t.shape[0], 3):
        raise VortaError(-1, f"t_emb [d_t] and w_r [heads, d_t, 3] expected, got {t.shape} and {w.shape}")
    heads, d_t = w.shape[0], t.shape[0]
    alpha = np.empty((heads, 3), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    _check(load_library().vorta_router_gates(t.ctypes.data_as(fp), w.ctypes.data_as(fp), d_t, heads,
                                             alpha.ctypes.data_as(fp)))
    return alpha


def vorta_route_select(alpha) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    if a.ndim != 2 or a.shape[1] != 3:
        raise VortaError(-1, f"alpha [heads, 3] expected, got {a.shape}")
    routes = np.empty(a.shape[0], dtype=np.uint8)
    _check(load_library().vorta_route_select(a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                             ctypes.c_int32(a.shape[0]), _u8p(routes)))
    return routes


def vorta_router_device(t_emb: torch.Tensor, w_r: torch.Tensor, alpha: torch.Tensor = None,
                        routes: torch.Tensor = None, routes_host: torch.Tensor = None, stream=None):
    """t_emb: device float32 [n_steps, d_t]; w_r: device float32 [heads, d_t, 3].  Returns
    (alpha [n_steps, heads, 3], routes uint8 [n_steps, heads]) on the device; routes_host (a
    CPU uint8 tensor of the same shape, pinned for an asynchronous copy) is filled once the
    stream has been synchronised."""
    for name, t in (("t_emb", t_emb), ("w_r", w_r)):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
            raise VortaError(-1, f"{name}: contiguous float32 device tensor expected")
    if t_emb.dim() != 2 or w_r.dim() != 3 or w_r.shape[1] != t_emb.shape[1] or w_r.shape[2] != 3 \
            or w_r.device != t_emb.device:
        raise VortaError(-2, f"t_emb [n_steps, d_t] and w_r [heads, d_t, 3] on one device expected, got "
                             f"{tuple(t_emb.shape)} and {tuple(w_r.shape)}")
    n_steps, d_t = t_emb.shape
    heads = w_r.shape[0]
    if alpha is None:
        alpha = torch.empty(n_steps, heads, 3, dtype=torch.float32, device=t_emb.device)
    if routes is None:
        routes = torch.empty(n_steps, heads, dtype=torch.uint8, device=t_emb.device)
    for name, t, shape, dt in (("alpha", alpha, (n_steps, heads, 3), torch.float32),
                               ("routes", routes, (n_steps, heads), torch.uint8)):
        if not t.is_cuda or t.device != t_emb.device or t.dtype != dt or tuple(t.shape) != shape or not t.is_contiguous():
            raise VortaError(-2, f"{name}: contiguous {dt} device tensor of shape {shape} expected")
    host_ptr = ctypes.c_void_p(0)
    if routes_host is not None:
        if routes_host.is_cuda or routes_host.dtype != torch.uint8 or tuple(routes_host.shape) != (n_steps, heads) \
                or not routes_host.is_contiguous():
            raise VortaError(-2, f"routes_host: contiguous uint8 CPU tensor of shape {(n_steps, heads)} expected")
        host_ptr = ctypes.c_void_p(routes_host.data_ptr())
    _check(load_library().vorta_router_device(_ptr(t_emb), _ptr(w_r), n_steps, d_t, heads, _ptr(alpha), _ptr(routes),
                                              host_ptr, _stream(stream)))
    return alpha, routes


# ---- device passes -------------------------------------------------------------------------

def _count(routes: np.ndarray, r: int) -> int:
    return int((routes == r).sum())


def vorta_plan_upload(plan: Plan):
    _check(load_library().vorta_plan_upload(plan.handle))


def vorta_reorder_to_tiles(plan: Plan, src: torch.Tensor, routes, dst: torch.Tensor = None, stream=None):
    r = _routes(routes, plan)
    if dst is None:
        dst = torch.empty(_count(r, 1), plan.n_tokens, plan.head_dim, dtype=src.dtype, device=src.device)
    _check_tensors(plan, src=plan._user(src), dst=plan._tiled(dst, _count(r, 1)))
    _check(load_library().vorta_reorder_to_tiles(plan.handle, _ptr(src), _u8p(r), _ptr(dst), _stream(stream)))
    return dst


def vorta_reorder_from_tiles(plan: Plan, src: torch.Tensor, routes, dst: torch.Tensor, stream=None):
    r = _routes(routes, plan)
    _check_tensors(plan, src=plan._tiled(src, _count(r, 1)), dst=plan._user(dst))
    _check(load_library().vorta_reorder_from_tiles(plan.handle, _ptr(src), _u8p(r), _ptr(dst), _stream(stream)))
    return dst


def vorta_bcs_build_index(plan: Plan, feat: torch.Tensor, routes, keep_idx=None, assign=None, stream=None,
                          feat_head_stride: int = VORTA_FEAT_USER_LAYOUT):
    """feat: a user-layout tensor (feat_head_stride = VORTA_FEAT_USER_LAYOUT), one [L or N, d] array
    shared by all heads (0), or [heads, rows, d] with feat_head_stride = rows * d."""
    r = _routes(routes, plan)
    n = _count(r, 2)
    if keep_idx is None:
        keep_idx = torch.empty(n, plan.n_core, dtype=torch.int32, device=feat.device)
    if assign is None:
        assign = torch.empty(n, plan.n_video, dtype=torch.int32, device=feat.device)
    if feat_head_stride == VORTA_FEAT_USER_LAYOUT:
        feat_spec = plan._user(feat)
    elif feat_head_stride == 0:
        if feat.dim() != 2 or feat.shape[0] < plan.n_video:
            raise VortaError(-2, f"feat: shape {tuple(feat.shape)}, a shared feature needs [>= {plan.n_video}, {plan.head_dim}]")
        feat_spec = (feat, (feat.shape[0], plan.head_dim), plan.torch_dtype)
    else:
        if feat.dim() != 3 or feat.shape[1] < plan.n_video or feat_head_stride != feat.shape[1] * plan.head_dim:
            raise VortaError(-2, f"feat: shape {tuple(feat.shape)} with head stride {feat_head_stride}: "
                                 f"[heads, rows >= {plan.n_video}, {plan.head_dim}] and stride rows * head_dim expected")
        feat_spec = (feat, (plan.heads, feat.shape[1], plan.head_dim), plan.torch_dtype)
    _check_tensors(plan, feat=feat_spec, keep_idx=(keep_idx, (n, plan.n_core), torch.int32),
                   assign=(assign, (n, plan.n_video), torch.int32))
    _check(load_library().vorta_bcs_build_index(plan.handle, _ptr(feat), ctypes.c_int64(feat_head_stride), _u8p(r),
                                                _ptr(keep_idx), _ptr(assign), _stream(stream)))
    return keep_idx, assign


def vorta_bcs_select_pool(plan: Plan, q, k, v, routes, keep_idx=None, assign=None, q_c=None, k_c=None, v_c=None,
                          stream=None):
    """Index on K and pooled Q, K, V in one call; returns (keep_idx, assign, q_c, k_c, v_c)."""
    r = _routes(routes, plan)
    n = _count(r, 2)
    dev = q.device
    if keep_idx is None:
        keep_idx = torch.empty(n, plan.n_core, dtype=torch.int32, device=dev)
    if assign is None:
        assign = torch.empty(n, plan.n_video, dtype=torch.int32, device=dev)
    q_c, k_c, v_c = (t if t is not None else torch.empty(n, plan.n_core_tokens, plan.head_dim, dtype=plan.torch_dtype, device=dev)
                     for t in (q_c, k_c, v_c))
    _check_tensors(plan, q=plan._user(q), k=plan._user(k), v=plan._user(v),
                   keep_idx=(keep_idx, (n, plan.n_core), torch.int32), assign=(assign, (n, plan.n_video), torch.int32),
                   q_c=plan._core(q_c, n), k_c=plan._core(k_c, n), v_c=plan._core(v_c, n))
    _check(load_library().vorta_bcs_select_pool(plan.handle, _ptr(q), _ptr(k), _ptr(v), _u8p(r), _ptr(keep_idx),
                                                _ptr(assign), _ptr(q_c), _ptr(k_c), _ptr(v_c), _stream(stream)))
    return keep_idx, assign, q_c, k_c, v_c


def vorta_rope_apply(plan: Plan, src: torch.Tensor, routes, dst: torch.Tensor = None, stream=None):
    """Rows of the heads on routes 0 and 1, turned by the plan's rotary embedding (other heads'
    rows of dst are left as they are: a fresh dst holds whatever torch.empty_like gives)."""
    r = _routes(routes, plan)
    if dst is None:
        dst = torch.empty_like(src)
    _check_tensors(plan, src=plan._user(src), dst=plan._user(dst))
    _check(load_library().vorta_rope_apply(plan.handle, _ptr(src), _u8p(r), _ptr(dst), _stream(stream)))
    return dst


def vorta_bcs_pool(plan: Plan, src: torch.Tensor, routes, keep_idx, assign, dst=None, stream=None, rotate=False):
    r = _routes(routes, plan)
    n = _count(r, 2)
    if dst is None:
        dst = torch.empty(n, plan.n_core_tokens, plan.head_dim, dtype=src.dtype, device=src.device)
    _check_tensors(plan, src=plan._user(src), keep_idx=(keep_idx, (n, plan.n_core), torch.int32),
                   assign=(assign, (n, plan.n_video), torch.int32), dst=plan._core(dst, n))
    _check(load_library().vorta_bcs_pool(plan.handle, _ptr(src), _u8p(r), _ptr(keep_idx), _ptr(assign),
                                         ctypes.c_int32(1 if rotate else 0), _ptr(dst), _stream(stream)))
    return dst


def vorta_attention_routed(plan: Plan, routes, *, q=None, k=None, v=None, out=None, q_t=None, k_t=None,
                           v_t=None, o_t=None, q_c=None, k_c=None, v_c=None, o_c=None, stream=None):
    r = _routes(routes, plan)
    n_win, n_lr = _count(r, 1), _count(r, 2)
    _check_tensors(plan, q=plan._user(q), k=plan._user(k), v=plan._user(v), out=plan._user(out),
                   q_t=plan._tiled(q_t, n_win), k_t=plan._tiled(k_t, n_win), v_t=plan._tiled(v_t, n_win),
                   o_t=plan._tiled(o_t, n_win), q_c=plan._core(q_c, n_lr), k_c=plan._core(k_c, n_lr),
                   v_c=plan._core(v_c, n_lr), o_c=plan._core(o_c, n_lr))
    io = vorta_attn_io(*[_ptr(t).value for t in (q, k, v, out, q_t, k_t, v_t, o_t, q_c, k_c, v_c, o_c)])
    _check(load_library().vorta_attention_routed(plan.handle, _u8p(r), ctypes.byref(io), _stream(stream)))


def vorta_scatter_back(plan: Plan, routes, o_t, o_c, assign, out: torch.Tensor, stream=None):
    r = _routes(routes, plan)
    n_win, n_lr = _count(r, 1), _count(r, 2)
    _check_tensors(plan, o_t=plan._tiled(o_t, n_win), o_c=plan._core(o_c, n_lr),
                   assign=(assign, (n_lr, plan.n_video), torch.int32), out=plan._user(out))
    _check(load_library().vorta_scatter_back(plan.handle, _u8p(r), _ptr(o_t), _ptr(o_c), _ptr(assign), _ptr(out),
                                             _stream(stream)))
    return out


def vorta_workspace_bytes(plan: Plan, routes) -> int:
    r = _routes(routes, plan)
    n = ctypes.c_size_t()
    _check(load_library().vorta_workspace_bytes(plan.handle, _u8p(r), ctypes.byref(n)))
    return n.value


def vorta_workspace_layout(plan: Plan, routes) -> Sequence[int]:
    r = _routes(routes, plan)
    off = (ctypes.c_size_t * 12)()
    _check(load_library().vorta_workspace_layout(plan.handle, _u8p(r), off))
    return list(off)


def vorta_routed_attention_layer(plan: Plan, q, k, v, routes, out=None, workspace=None, stream=None):
    r = _routes(routes, plan)
    _check_tensors(plan, q=plan._user(q), k=plan._user(k), v=plan._user(v))
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(vorta_workspace_bytes(plan, r), dtype=torch.uint8, device=q.device)
    _check_tensors(plan, q=plan._user(q), out=plan._user(out))
    _check_workspace(workspace)
    if workspace.device != q.device:
        raise VortaError(-1, f"workspace is on {workspace.device}, q on {q.device}")
    _check(load_library().vorta_routed_attention_layer(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), _u8p(r), _ptr(out), _ptr(workspace),
        ctypes.c_size_t(workspace.numel()), _stream(stream)))
    return out


def vorta_routed_attention_layer_static(plan: Plan, q, k, v, routes, out, stream=None):
    """The layer call for callers that cannot allocate: no workspace argument (the library's
    static scratch is used), `out` must be given, vorta_plan_upload(plan) must have been called."""
    r = _routes(routes, plan)
    _check_tensors(plan, q=plan._user(q), k=plan._user(k), v=plan._user(v), out=plan._user(out))
    _check(load_library().vorta_routed_attention_layer_static(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), _u8p(r), _ptr(out), _stream(stream)))
    return out


def vorta_soft_mixture_workspace_bytes(plan: Plan) -> int:
    n = ctypes.c_size_t()
    _check(load_library().vorta_soft_mixture_workspace_bytes(plan.handle, ctypes.byref(n)))
    return n.value


def vorta_soft_mixture_layer(plan: Plan, q, k, v, alpha, out=None, workspace=None, stream=None):
    a = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    if a.shape != (plan.heads, 3):
        raise VortaError(-1, f"alpha has shape {a.shape}, the plan needs ({plan.heads}, 3)")
    _check_tensors(plan, q=plan._user(q), k=plan._user(k), v=plan._user(v))
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(vorta_soft_mixture_workspace_bytes(plan), dtype=torch.uint8, device=q.device)
    _check_tensors(plan, q=plan._user(q), out=plan._user(out))
    _check_workspace(workspace)
    if workspace.device != q.device:
        raise VortaError(-1, f"workspace is on {workspace.device}, q on {q.device}")
    _check(load_library().vorta_soft_mixture_layer(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _ptr(out),
        _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(stream)))
    return out
