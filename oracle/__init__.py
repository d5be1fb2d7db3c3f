"""ctypes front end of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never touches the GPU library and the GPU library never
touches it.  Arrays are numpy, host memory; bf16 tensors travel as uint16 bit
patterns, fp32 tensors as float32.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

F32, BF16, FP8_E4M3 = 0, 1, 2
REDUCE_MAX, REDUCE_MEAN = 0, 1
HEADS_SEPARATE, HEADS_JOINT = 0, 1


class _Params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("ctx_len", ctypes.c_int32), ("group_size", ctypes.c_int32), ("n_select", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32), ("meta_dtype", ctypes.c_int32),
        ("reduce", ctypes.c_int32), ("head_mode", ctypes.c_int32), ("ctx_capacity", ctypes.c_int32),
        ("n_threads", ctypes.c_int32), ("meta_scale", ctypes.c_double),
        ("softmax_scale", ctypes.c_double), ("meta_scales", ctypes.c_void_p),
    ]


@dataclass
class Shape:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rank: int
    ctx_len: int
    group_size: int
    n_select: int
    kv_dtype: int = F32
    meta_dtype: int = F32
    reduce: int = REDUCE_MAX
    n_threads: int = 1
    softmax_scale: float = 0.0
    head_mode: int = HEADS_SEPARATE
    ctx_capacity: int = 0      # rows allocated per problem in K, V, K_lr (0: ctx_len)
    meta_scale: float = 0.0    # K_lr is stored divided by this (0: 1)
    meta_scales: object = None  # optional float64 array, one scale per selection set (overrides meta_scale)

    def __post_init__(self):
        if self.meta_scales is not None:     # held as a contiguous float64 array: the C struct takes its address
            a = np.ascontiguousarray(self.meta_scales, dtype=np.float64)
            if a.shape != self.sets:
                raise ValueError(f"meta_scales: expected shape {self.sets}, got {a.shape}")
            self.meta_scales = a

    def _c(self) -> _Params:
        ptr = None if self.meta_scales is None else self.meta_scales.ctypes.data_as(ctypes.c_void_p)
        return _Params(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.rank,
                       self.ctx_len, self.group_size, self.n_select, self.kv_dtype,
                       self.meta_dtype, self.reduce, self.head_mode, self.ctx_capacity,
                       self.n_threads, self.meta_scale, self.softmax_scale, ptr)

    @property
    def rows(self) -> int:
        """Rows held per problem by K, V and K_lr."""
        return self.ctx_capacity or self.ctx_len

    @property
    def n_groups(self) -> int:
        return self.ctx_len // self.group_size

    @property
    def sets(self) -> tuple:
        """Leading axes of the per-selection-set tensors (K_lr, idx, gs, s)."""
        return (self.batch,) if self.head_mode == HEADS_JOINT else (self.batch, self.n_kv_heads)


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        _lib = ctypes.CDLL(path)
        vp, pp = ctypes.c_void_p, ctypes.POINTER(_Params)
        _lib.oracle_build_metadata.argtypes = [pp, vp, vp, vp, vp]
        _lib.oracle_predict_select.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
        _lib.oracle_sparse_attn.argtypes = [pp, vp, vp, vp, vp, vp]
        i32 = ctypes.c_int32
        _lib.oracle_sparse_attn_rb.argtypes = [pp, vp, vp, vp, vp, vp, vp, i32, i32, vp]
        _lib.oracle_build_metadata_rows.argtypes = [pp, vp, vp, vp, vp, i32, i32]
        _lib.oracle_sparse_attn_paged.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i32, vp]
        _lib.oracle_selection_overlap.argtypes = [pp, vp, vp, vp]
        _lib.oracle_sparse_attn_paged.restype = ctypes.c_int
        _lib.oracle_selection_overlap.restype = ctypes.c_int
        _lib.oracle_dense_attn.argtypes = [pp, vp, vp, vp, vp]
        _lib.oracle_round_to_bf16.argtypes = [ctypes.c_double]
        _lib.oracle_round_to_bf16.restype = ctypes.c_uint16
        _lib.oracle_round_to_fp8_e4m3.argtypes = [ctypes.c_double]
        _lib.oracle_round_to_fp8_e4m3.restype = ctypes.c_uint8
        _lib.oracle_fp8_e4m3_value.argtypes = [ctypes.c_uint8]
        _lib.oracle_fp8_e4m3_value.restype = ctypes.c_double
        for f in (_lib.oracle_build_metadata, _lib.oracle_predict_select, _lib.oracle_sparse_attn,
                  _lib.oracle_dense_attn, _lib.oracle_sparse_attn_rb, _lib.oracle_build_metadata_rows):
            f.restype = ctypes.c_int
    return _lib


def _np_dtype(code: int):
    return {F32: np.float32, BF16: np.uint16, FP8_E4M3: np.uint8}[code]


def _arr(x, dtype, shape, name):
    a = np.ascontiguousarray(x)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"{name}: expected dtype {np.dtype(dtype)}, got {a.dtype}")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


def build_metadata(sh: Shape, K, A, want_exact: bool = False):
    """K_lr = K . A, rounded once to meta_dtype.  Returns storage array
    [B,H_kv,N,r] ([B,N,r] in joint mode) (and the unrounded fp64 products if want_exact)."""
    K = _arr(K, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_kv_heads, sh.rows, sh.head_dim), "K")
    A = _arr(A, np.float32, (sh.n_kv_heads, sh.head_dim, sh.rank), "A")
    # rows beyond ctx_len (capacity) are not computed: they come back as zeros
    out = np.zeros(sh.sets + (sh.rows, sh.rank), dtype=_np_dtype(sh.meta_dtype))
    exact = np.zeros(out.shape, dtype=np.float64) if want_exact else None
    c = sh._c()
    _check(lib().oracle_build_metadata(ctypes.byref(c), _ptr(K), _ptr(A), _ptr(out), _ptr(exact)),
           "oracle_build_metadata")
    return (out, exact) if want_exact else out


def build_metadata_rows(sh: Shape, K, A, K_lr, first_row: int, n_rows: int, exact=None):
    """Metadata of token rows [first_row, first_row + n_rows) written into K_lr in place
    (and the unrounded products into `exact`, if given)."""
    K = _arr(K, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_kv_heads, sh.rows, sh.head_dim), "K")
    A = _arr(A, np.float32, (sh.n_kv_heads, sh.head_dim, sh.rank), "A")
    if not (isinstance(K_lr, np.ndarray) and K_lr.flags.c_contiguous and K_lr.flags.writeable
            and K_lr.dtype == np.dtype(_np_dtype(sh.meta_dtype))
            and K_lr.shape == sh.sets + (sh.rows, sh.rank)):
        raise ValueError("K_lr: need a writable contiguous array of the metadata shape and dtype")
    if exact is not None and not (exact.dtype == np.float64 and exact.shape == K_lr.shape
                                  and exact.flags.c_contiguous):
        raise ValueError("exact: need a contiguous float64 array of the metadata shape")
    c = sh._c()
    _check(lib().oracle_build_metadata_rows(ctypes.byref(c), _ptr(K), _ptr(A), _ptr(K_lr),
                                            _ptr(exact), int(first_row), int(n_rows)),
           "oracle_build_metadata_rows")


def predict_select(sh: Shape, q, K_lr, A):
    """Returns dict(idx [B,H_kv,M] int32 ascending, gs [B,H_kv,NG] f64,
    s [B,H_kv,N] f64, boundary [B,H_kv,2] f64); no H_kv axis in joint mode."""
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    K_lr = _arr(K_lr, _np_dtype(sh.meta_dtype), sh.sets + (sh.rows, sh.rank), "K_lr")
    A = _arr(A, np.float32, (sh.n_kv_heads, sh.head_dim, sh.rank), "A")
    P = sh.sets
    idx = np.empty(P + (sh.n_select,), dtype=np.int32)
    gs = np.empty(P + (sh.n_groups,), dtype=np.float64)
    s = np.empty(P + (sh.ctx_len,), dtype=np.float64)
    bnd = np.empty(P + (2,), dtype=np.float64)
    c = sh._c()
    _check(lib().oracle_predict_select(ctypes.byref(c), _ptr(q), _ptr(K_lr), _ptr(A), _ptr(idx),
                                       _ptr(gs), _ptr(s), _ptr(bnd)), "oracle_predict_select")
    return {"idx": idx, "gs": gs, "s": s, "boundary": bnd}


def sparse_attn(sh: Shape, q, K, V, idx, rb_K=None, rb_V=None, rb_len: int = 0):
    """Attention over the selected groups (and, if given, the first rb_len tokens of the
    rolling buffer rb_K / rb_V [B,H_kv,capacity,d])."""
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    shape_kv = (sh.batch, sh.n_kv_heads, sh.rows, sh.head_dim)
    K = _arr(K, _np_dtype(sh.kv_dtype), shape_kv, "K")
    V = _arr(V, _np_dtype(sh.kv_dtype), shape_kv, "V")
    idx = _arr(idx, np.int32, sh.sets + (sh.n_select,), "idx")
    out = np.empty((sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    c = sh._c()
    cap = 0
    if rb_K is not None:
        cap = rb_K.shape[2]
        shape_rb = (sh.batch, sh.n_kv_heads, cap, sh.head_dim)
        rb_K = _arr(rb_K, _np_dtype(sh.kv_dtype), shape_rb, "rb_K")
        rb_V = _arr(rb_V, _np_dtype(sh.kv_dtype), shape_rb, "rb_V")
    _check(lib().oracle_sparse_attn_rb(ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                       _ptr(rb_K), _ptr(rb_V), int(rb_len), int(cap), _ptr(out)),
           "oracle_sparse_attn_rb")
    return out


def sparse_attn_paged(sh: Shape, q, K_pool, V_pool, slot_table, idx, rb_K=None, rb_V=None, rb_len: int = 0):
    """Attention over the selected groups read through a mapping table: K_pool, V_pool
    [n_slots, G, d], slot_table [B, H_kv, NG] int32 (logical group -> slot)."""
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    n_slots = K_pool.shape[0]
    shape_pool = (n_slots, sh.group_size, sh.head_dim)
    K_pool = _arr(K_pool, _np_dtype(sh.kv_dtype), shape_pool, "K_pool")
    V_pool = _arr(V_pool, _np_dtype(sh.kv_dtype), shape_pool, "V_pool")
    slot_table = _arr(slot_table, np.int32, (sh.batch, sh.n_kv_heads, sh.n_groups), "slot_table")
    idx = _arr(idx, np.int32, sh.sets + (sh.n_select,), "idx")
    out = np.empty((sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    cap = 0
    if rb_K is not None:
        cap = rb_K.shape[2]
        shape_rb = (sh.batch, sh.n_kv_heads, cap, sh.head_dim)
        rb_K = _arr(rb_K, _np_dtype(sh.kv_dtype), shape_rb, "rb_K")
        rb_V = _arr(rb_V, _np_dtype(sh.kv_dtype), shape_rb, "rb_V")
    c = sh._c()
    _check(lib().oracle_sparse_attn_paged(ctypes.byref(c), _ptr(q), _ptr(K_pool), _ptr(V_pool),
                                          _ptr(slot_table), int(n_slots), _ptr(idx), _ptr(rb_K),
                                          _ptr(rb_V), int(rb_len), int(cap), _ptr(out)),
           "oracle_sparse_attn_paged")
    return out


def selection_overlap(sh: Shape, idx_prev, idx_cur):
    """Number of groups common to two selections, per selection set (int32 array)."""
    idx_prev = _arr(idx_prev, np.int32, sh.sets + (sh.n_select,), "idx_prev")
    idx_cur = _arr(idx_cur, np.int32, sh.sets + (sh.n_select,), "idx_cur")
    out = np.empty(sh.sets, dtype=np.int32)
    c = sh._c()
    _check(lib().oracle_selection_overlap(ctypes.byref(c), _ptr(idx_prev), _ptr(idx_cur), _ptr(out)),
           "oracle_selection_overlap")
    return out


def dense_attn(sh: Shape, q, K, V):
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    shape_kv = (sh.batch, sh.n_kv_heads, sh.rows, sh.head_dim)
    K = _arr(K, _np_dtype(sh.kv_dtype), shape_kv, "K")
    V = _arr(V, _np_dtype(sh.kv_dtype), shape_kv, "V")
    out = np.empty((sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    c = sh._c()
    _check(lib().oracle_dense_attn(ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(out)),
           "oracle_dense_attn")
    return out


def round_to_bf16(x: float) -> int:
    return int(lib().oracle_round_to_bf16(float(x)))


def round_to_fp8_e4m3(x: float) -> int:
    return int(lib().oracle_round_to_fp8_e4m3(float(x)))


def fp8_e4m3_value(code: int) -> float:
    return float(lib().oracle_fp8_e4m3_value(int(code)))
