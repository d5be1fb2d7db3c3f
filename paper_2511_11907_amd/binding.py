"""ctypes binding of libkvswap_hip.so (declared in include/kvswap_hip.h).

Functions carry the names of the C entry points and take torch tensors that
already live on the GPU; this layer checks dtype / shape / contiguity, passes
raw device pointers and the current HIP stream, and raises KvsError on any
non-zero status.  torch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

from . import build as _build

KVS_F32, KVS_BF16, KVS_FP8_E4M3 = 0, 1, 2
KVS_REDUCE_MAX, KVS_REDUCE_MEAN = 0, 1
KVS_HEADS_SEPARATE, KVS_HEADS_JOINT = 0, 1
KVS_STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = (
    "kvs_workspace_bytes", "kvs_workspace_init", "kvs_workspace_check", "kvs_set_wait_limit",
    "kvs_check_params", "kvs_build_metadata",
    "kvs_build_metadata_rows", "kvs_append_group", "kvs_predict_select",
    "kvs_predict_scores", "kvs_select_topk",
    "kvs_sparse_decode_attn", "kvs_sparse_decode_attn_rb", "kvs_sparse_decode_attn_paged",
    "kvs_selection_overlap", "kvs_decode_step", "kvs_decode_step_rb", "kvs_decode_step_static",
    "kvs_decode_step_single_launch", "kvs_attend_select_next", "kvs_attend_select_next_rb",
    "kvs_status_str", "kvs_version", "kvs_last_device_error",
)


class KvsError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        detail = f": {kvs_last_device_error()}" if status == 6 else ""
        super().__init__(f"{what}: status {status} ({kvs_status_str(status)}){detail}")


class _CParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("ctx_len", ctypes.c_int32), ("group_size", ctypes.c_int32), ("n_select", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32), ("meta_dtype", ctypes.c_int32), ("reduce", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("head_mode", ctypes.c_int32),
        ("meta_scale", ctypes.c_float), ("ctx_capacity", ctypes.c_int32),
        ("meta_scales", ctypes.c_void_p),
    ]


@dataclass
class Params:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rank: int
    ctx_len: int
    group_size: int
    n_select: int
    kv_dtype: int = KVS_BF16
    meta_dtype: int = KVS_BF16
    reduce: int = KVS_REDUCE_MAX
    softmax_scale: float = 0.0
    head_mode: int = KVS_HEADS_SEPARATE
    ctx_capacity: int = 0      # rows allocated per problem in K, V, K_lr (0: ctx_len)
    meta_scale: float = 0.0    # K_lr is stored divided by this (0: 1)
    meta_scales: object = None  # optional fp32 GPU tensor of shape `sets`: one scale per selection set

    def _c(self) -> _CParams:
        ptr = None
        if self.meta_scales is not None:
            t = self.meta_scales
            import torch
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == self.sets):
                raise ValueError(f"meta_scales must be a contiguous fp32 GPU tensor of shape {self.sets}")
            ptr = ctypes.c_void_p(t.data_ptr())
        return _CParams(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.rank,
                        self.ctx_len, self.group_size, self.n_select, self.kv_dtype,
                        self.meta_dtype, self.reduce, self.softmax_scale, self.head_mode,
                        self.meta_scale, self.ctx_capacity, ptr)

    @property
    def rows(self) -> int:
        """Rows held per problem by K, V and K_lr."""
        return self.ctx_capacity or self.ctx_len

    @property
    def n_groups(self) -> int:
        return self.ctx_len // self.group_size

    @property
    def sets(self) -> tuple:
        """Leading axes of K_lr, idx and group_scores: (B, H_kv), or (B,) in joint-head mode."""
        return (self.batch,) if self.head_mode == KVS_HEADS_JOINT else (self.batch, self.n_kv_heads)


_lib = None


def library_path() -> str:
    """The in-tree library, unless KVSWAP_HIP_LIBRARY names another build of it."""
    return os.environ.get("KVSWAP_HIP_LIBRARY") or _build.LIB


def load_library() -> ctypes.CDLL:
    """Load the built library; build it first only if no library is there.
    Raises if it cannot be built or loaded -- there is no other code path."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        _build.build()
    # torch ships its own HIP runtime (same soname as the system one).  Importing torch
    # first makes the loader resolve this library against that already-loaded runtime,
    # so the process has one runtime and device pointers mean the same thing to both.
    _torch()
    lib = ctypes.CDLL(path)
    vp, pp, sz = ctypes.c_void_p, ctypes.POINTER(_CParams), ctypes.c_size_t
    lib.kvs_workspace_bytes.argtypes = [pp]
    lib.kvs_workspace_bytes.restype = sz
    lib.kvs_workspace_init.argtypes = [pp, vp, sz, vp]
    lib.kvs_workspace_init.restype = ctypes.c_int
    lib.kvs_workspace_check.argtypes = [pp, vp, sz, vp]
    lib.kvs_workspace_check.restype = ctypes.c_int
    lib.kvs_set_wait_limit.argtypes = [ctypes.c_int32]
    lib.kvs_set_wait_limit.restype = None
    lib.kvs_check_params.argtypes = [pp]
    lib.kvs_check_params.restype = ctypes.c_int
    lib.kvs_build_metadata.argtypes = [pp, vp, vp, vp, vp]
    lib.kvs_build_metadata.restype = ctypes.c_int
    i32 = ctypes.c_int32
    lib.kvs_build_metadata_rows.argtypes = [pp, vp, vp, vp, i32, i32, vp]
    lib.kvs_build_metadata_rows.restype = ctypes.c_int
    lib.kvs_append_group.argtypes = [pp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.kvs_append_group.restype = ctypes.c_int
    lib.kvs_sparse_decode_attn_rb.argtypes = [pp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.kvs_sparse_decode_attn_rb.restype = ctypes.c_int
    lib.kvs_sparse_decode_attn_paged.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.kvs_sparse_decode_attn_paged.restype = ctypes.c_int
    lib.kvs_selection_overlap.argtypes = [pp, vp, vp, vp, vp]
    lib.kvs_selection_overlap.restype = ctypes.c_int
    lib.kvs_decode_step_rb.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.kvs_decode_step_rb.restype = ctypes.c_int
    lib.kvs_predict_select.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_predict_select.restype = ctypes.c_int
    lib.kvs_predict_scores.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_predict_scores.restype = ctypes.c_int
    lib.kvs_select_topk.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.kvs_select_topk.restype = ctypes.c_int
    lib.kvs_sparse_decode_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_sparse_decode_attn.restype = ctypes.c_int
    lib.kvs_decode_step.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_decode_step.restype = ctypes.c_int
    lib.kvs_decode_step_single_launch.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_decode_step_single_launch.restype = ctypes.c_int
    lib.kvs_attend_select_next.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_attend_select_next.restype = ctypes.c_int
    lib.kvs_attend_select_next_rb.argtypes = [pp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.kvs_attend_select_next_rb.restype = ctypes.c_int
    lib.kvs_decode_step_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.kvs_decode_step_static.restype = ctypes.c_int
    lib.kvs_status_str.argtypes = [ctypes.c_int]
    lib.kvs_status_str.restype = ctypes.c_char_p
    lib.kvs_last_device_error.argtypes = []
    lib.kvs_last_device_error.restype = ctypes.c_char_p
    lib.kvs_version.argtypes = []
    lib.kvs_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


# ---- helpers ------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _dtype_of(code: int):
    torch = _torch()
    return {KVS_F32: torch.float32, KVS_BF16: torch.bfloat16, KVS_FP8_E4M3: torch.float8_e4m3fn}[code]


def _dev(t, dtype, shape, name):
    if t is None:
        raise ValueError(f"{name} is required")
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _ws(workspace):
    if workspace is None:
        return ctypes.c_void_p(0), 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, what: str):
    if status != 0:
        raise KvsError(status, what)


# ---- entry points ---------------------------------------------------------------
def kvs_status_str(status: int) -> str:
    return load_library().kvs_status_str(int(status)).decode()


def kvs_last_device_error() -> str:
    return load_library().kvs_last_device_error().decode()


def kvs_version() -> str:
    return load_library().kvs_version().decode()


def kvs_check_params(p: Params) -> int:
    c = p._c()
    return int(load_library().kvs_check_params(ctypes.byref(c)))


def kvs_workspace_bytes(p: Params) -> int:
    c = p._c()
    return int(load_library().kvs_workspace_bytes(ctypes.byref(c)))


def kvs_workspace_init(p: Params, workspace, stream=None) -> None:
    c = p._c()
    ws, nws = _ws(workspace)
    _check(load_library().kvs_workspace_init(ctypes.byref(c), ws, nws, _stream(stream)),
           "kvs_workspace_init")


def kvs_workspace_check(p: Params, workspace, stream=None) -> int:
    """Status code (0, or 6 if a wait inside kvs_decode_step ever ran out); synchronises the stream."""
    c = p._c()
    ws, nws = _ws(workspace)
    return int(load_library().kvs_workspace_check(ctypes.byref(c), ws, nws, _stream(stream)))


def kvs_set_wait_limit(polls: int) -> None:
    load_library().kvs_set_wait_limit(int(polls))


def _metadata_args(p: Params, K, A, K_lr):
    torch = _torch()
    kd, md = _dtype_of(p.kv_dtype), _dtype_of(p.meta_dtype)
    return (_dev(K, kd, (p.batch, p.n_kv_heads, p.rows, p.head_dim), "K"),
            _dev(A, torch.float32, (p.n_kv_heads, p.head_dim, p.rank), "A"),
            _dev(K_lr, md, p.sets + (p.rows, p.rank), "K_lr"))


def kvs_build_metadata(p: Params, K, A, K_lr, stream=None) -> None:
    c = p._c()
    st = load_library().kvs_build_metadata(ctypes.byref(c), *_metadata_args(p, K, A, K_lr), _stream(stream))
    _check(st, "kvs_build_metadata")


def kvs_build_metadata_rows(p: Params, K, A, K_lr, first_row: int, n_rows: int, stream=None) -> None:
    c = p._c()
    st = load_library().kvs_build_metadata_rows(ctypes.byref(c), *_metadata_args(p, K, A, K_lr),
                                                int(first_row), int(n_rows), _stream(stream))
    _check(st, "kvs_build_metadata_rows")


def _rb(p: Params, rb_K, rb_V, rb_len: int):
    """Rolling-buffer tensors [B,H_kv,capacity,d] -> (K pointer, V pointer, len, capacity)."""
    if rb_K is None or rb_V is None:
        if rb_len:
            raise ValueError("rb_len > 0 needs rb_K and rb_V")
        return ctypes.c_void_p(0), ctypes.c_void_p(0), 0, 0
    kd = _dtype_of(p.kv_dtype)
    if rb_K.dim() != 4:
        raise ValueError("rb_K must be [B, H_kv, capacity, d]")
    cap = int(rb_K.shape[2])
    shape = (p.batch, p.n_kv_heads, cap, p.head_dim)
    return _dev(rb_K, kd, shape, "rb_K"), _dev(rb_V, kd, shape, "rb_V"), int(rb_len), cap


def kvs_append_group(p: Params, rb_K, rb_V, K, V, A, K_lr, stream=None) -> None:
    torch = _torch()
    kd, md = _dtype_of(p.kv_dtype), _dtype_of(p.meta_dtype)
    c = p._c()
    rk, rv, _, cap = _rb(p, rb_K, rb_V, 0)
    kv_shape = (p.batch, p.n_kv_heads, p.rows, p.head_dim)
    st = load_library().kvs_append_group(
        ctypes.byref(c), rk, rv, cap,
        _dev(K, kd, kv_shape, "K"), _dev(V, kd, kv_shape, "V"),
        _dev(A, torch.float32, (p.n_kv_heads, p.head_dim, p.rank), "A"),
        _dev(K_lr, md, p.sets + (p.rows, p.rank), "K_lr"),
        _stream(stream))
    _check(st, "kvs_append_group")


def kvs_predict_select(p: Params, q, K_lr, A, idx, group_scores, workspace, stream=None) -> None:
    torch = _torch()
    kd, md = _dtype_of(p.kv_dtype), _dtype_of(p.meta_dtype)
    c = p._c()
    ws, nws = _ws(workspace)
    gs = ctypes.c_void_p(0) if group_scores is None else _dev(
        group_scores, torch.float32, p.sets + (p.n_groups,), "group_scores")
    st = load_library().kvs_predict_select(
        ctypes.byref(c),
        _dev(q, kd, (p.batch, p.n_q_heads, p.head_dim), "q"),
        _dev(K_lr, md, p.sets + (p.rows, p.rank), "K_lr"),
        _dev(A, torch.float32, (p.n_kv_heads, p.head_dim, p.rank), "A"),
        _dev(idx, torch.int32, p.sets + (p.n_select,), "idx"),
        gs, ws, nws, _stream(stream))
    _check(st, "kvs_predict_select")


def kvs_predict_scores(p: Params, q, K_lr, A, group_scores, workspace=None, stream=None) -> None:
    torch = _torch()
    kd, md = _dtype_of(p.kv_dtype), _dtype_of(p.meta_dtype)
    c = p._c()
    ws, nws = _ws(workspace)
    st = load_library().kvs_predict_scores(
        ctypes.byref(c),
        _dev(q, kd, (p.batch, p.n_q_heads, p.head_dim), "q"),
        _dev(K_lr, md, p.sets + (p.rows, p.rank), "K_lr"),
        _dev(A, torch.float32, (p.n_kv_heads, p.head_dim, p.rank), "A"),
        _dev(group_scores, torch.float32, p.sets + (p.n_groups,), "group_scores"),
        ws, nws, _stream(stream))
    _check(st, "kvs_predict_scores")


def kvs_select_topk(p: Params, group_scores, idx, workspace=None, stream=None) -> None:
    torch = _torch()
    c = p._c()
    ws, nws = _ws(workspace)
    st = load_library().kvs_select_topk(
        ctypes.byref(c),
        _dev(group_scores, torch.float32, p.sets + (p.n_groups,), "group_scores"),
        _dev(idx, torch.int32, p.sets + (p.n_select,), "idx"),
        ws, nws, _stream(stream))
    _check(st, "kvs_select_topk")


def _attn_args(p: Params, q, K, V, idx, out, workspace, stream):
    """(head, tail) argument lists shared by the attention entry points."""
    torch = _torch()
    kd = _dtype_of(p.kv_dtype)
    ws, nws = _ws(workspace)
    kv_shape = (p.batch, p.n_kv_heads, p.rows, p.head_dim)
    head = [_dev(q, kd, (p.batch, p.n_q_heads, p.head_dim), "q"),
            _dev(K, kd, kv_shape, "K"), _dev(V, kd, kv_shape, "V"),
            _dev(idx, torch.int32, p.sets + (p.n_select,), "idx")]
    tail = [_dev(out, kd, (p.batch, p.n_q_heads, p.head_dim), "out"), ws, nws, _stream(stream)]
    return head, tail


def kvs_sparse_decode_attn(p: Params, q, K, V, idx, out, workspace, stream=None) -> None:
    c = p._c()
    head, tail = _attn_args(p, q, K, V, idx, out, workspace, stream)
    _check(load_library().kvs_sparse_decode_attn(ctypes.byref(c), *head, *tail), "kvs_sparse_decode_attn")


def kvs_attend_select_next(p: Params, q, K, V, idx, out, next_group_scores, next_idx, workspace, stream=None) -> None:
    torch = _torch()
    c = p._c()
    head, tail = _attn_args(p, q, K, V, idx, out, workspace, stream)
    nxt = [_dev(next_group_scores, torch.float32, p.sets + (p.n_groups,), "next_group_scores"),
           _dev(next_idx, torch.int32, p.sets + (p.n_select,), "next_idx")]
    _check(load_library().kvs_attend_select_next(ctypes.byref(c), *head, tail[0], *nxt, *tail[1:]),
           "kvs_attend_select_next")


def kvs_attend_select_next_rb(p: Params, q, K, V, idx, rb_K, rb_V, rb_len, out, next_group_scores, next_idx,
                              workspace, stream=None) -> None:
    torch = _torch()
    c = p._c()
    head, tail = _attn_args(p, q, K, V, idx, out, workspace, stream)
    nxt = [_dev(next_group_scores, torch.float32, p.sets + (p.n_groups,), "next_group_scores"),
           _dev(next_idx, torch.int32, p.sets + (p.n_select,), "next_idx")]
    _check(load_library().kvs_attend_select_next_rb(ctypes.byref(c), *head, *_rb(p, rb_K, rb_V, rb_len), tail[0],
                                                    *nxt, *tail[1:]), "kvs_attend_select_next_rb")


def kvs_sparse_decode_attn_rb(p: Params, q, K, V, idx, rb_K, rb_V, rb_len, out, workspace, stream=None) -> None:
    c = p._c()
    head, tail = _attn_args(p, q, K, V, idx, out, workspace, stream)
    _check(load_library().kvs_sparse_decode_attn_rb(ctypes.byref(c), *head, *_rb(p, rb_K, rb_V, rb_len), *tail),
           "kvs_sparse_decode_attn_rb")


def kvs_sparse_decode_attn_paged(p: Params, q, K_pool, V_pool, slot_table, idx, out, workspace,
                                 rb_K=None, rb_V=None, rb_len: int = 0, stream=None) -> None:
    """K_pool, V_pool [n_slots, G, d]; slot_table [B, H_kv, N/G] int32 (logical group -> slot)."""
    torch = _torch()
    kd = _dtype_of(p.kv_dtype)
    c = p._c()
    ws, nws = _ws(workspace)
    if K_pool is None or K_pool.dim() != 3:
        raise ValueError("K_pool must be [n_slots, G, d]")
    n_slots = int(K_pool.shape[0])
    pool_shape = (n_slots, p.group_size, p.head_dim)
    st = load_library().kvs_sparse_decode_attn_paged(
        ctypes.byref(c),
        _dev(q, kd, (p.batch, p.n_q_heads, p.head_dim), "q"),
        _dev(K_pool, kd, pool_shape, "K_pool"), _dev(V_pool, kd, pool_shape, "V_pool"),
        _dev(slot_table, torch.int32, (p.batch, p.n_kv_heads, p.n_groups), "slot_table"), n_slots,
        _dev(idx, torch.int32, p.sets + (p.n_select,), "idx"),
        *_rb(p, rb_K, rb_V, rb_len),
        _dev(out, kd, (p.batch, p.n_q_heads, p.head_dim), "out"), ws, nws, _stream(stream))
    _check(st, "kvs_sparse_decode_attn_paged")


def kvs_selection_overlap(p: Params, idx_prev, idx_cur, common, stream=None) -> None:
    torch = _torch()
    c = p._c()
    st = load_library().kvs_selection_overlap(
        ctypes.byref(c),
        _dev(idx_prev, torch.int32, p.sets + (p.n_select,), "idx_prev"),
        _dev(idx_cur, torch.int32, p.sets + (p.n_select,), "idx_cur"),
        _dev(common, torch.int32, p.sets, "common"), _stream(stream))
    _check(st, "kvs_selection_overlap")


def _step_args(p: Params, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream):
    """(head, tail) argument lists shared by the whole-step entry points."""
    torch = _torch()
    kd, md = _dtype_of(p.kv_dtype), _dtype_of(p.meta_dtype)
    ws, nws = _ws(workspace)
    kv_shape = (p.batch, p.n_kv_heads, p.rows, p.head_dim)
    gs = ctypes.c_void_p(0) if group_scores is None else _dev(
        group_scores, torch.float32, p.sets + (p.n_groups,), "group_scores")
    head = [_dev(q, kd, (p.batch, p.n_q_heads, p.head_dim), "q"),
            _dev(K_lr, md, p.sets + (p.rows, p.rank), "K_lr"),
            _dev(A, torch.float32, (p.n_kv_heads, p.head_dim, p.rank), "A"),
            _dev(K, kd, kv_shape, "K"), _dev(V, kd, kv_shape, "V")]
    tail = [_dev(idx, torch.int32, p.sets + (p.n_select,), "idx"), gs,
            _dev(out, kd, (p.batch, p.n_q_heads, p.head_dim), "out"), ws, nws, _stream(stream)]
    return head, tail


def kvs_decode_step(p: Params, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream=None) -> None:
    c = p._c()
    head, tail = _step_args(p, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream)
    _check(load_library().kvs_decode_step(ctypes.byref(c), *head, *tail), "kvs_decode_step")


def kvs_decode_step_single_launch(p: Params, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream=None) -> None:
    c = p._c()
    head, tail = _step_args(p, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream)
    _check(load_library().kvs_decode_step_single_launch(ctypes.byref(c), *head, *tail), "kvs_decode_step_single_launch")


def kvs_decode_step_static(p: Params, q, K_lr, A, K, V, idx, group_scores, out, stream=None) -> None:
    """kvs_decode_step on the library's own static scratch memory (no workspace argument)."""
    c = p._c()
    head, tail = _step_args(p, q, K_lr, A, K, V, idx, group_scores, out, None, stream)
    # tail = [idx, group_scores, out, workspace, workspace_bytes, stream]
    _check(load_library().kvs_decode_step_static(ctypes.byref(c), *head, *tail[:3], tail[5]),
           "kvs_decode_step_static")


def kvs_decode_step_rb(p: Params, q, K_lr, A, K, V, rb_K, rb_V, rb_len, idx, group_scores, out,
                       workspace, stream=None) -> None:
    c = p._c()
    head, tail = _step_args(p, q, K_lr, A, K, V, idx, group_scores, out, workspace, stream)
    _check(load_library().kvs_decode_step_rb(ctypes.byref(c), *head, *_rb(p, rb_K, rb_V, rb_len), *tail),
           "kvs_decode_step_rb")
