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

F32, BF16 = 0, 1
REDUCE_MAX, REDUCE_MEAN = 0, 1
HEADS_SEPARATE, HEADS_JOINT = 0, 1


class _Params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("ctx_len", ctypes.c_int32), ("group_size", ctypes.c_int32), ("n_select", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32), ("meta_dtype", ctypes.c_int32),
        ("reduce", ctypes.c_int32), ("head_mode", ctypes.c_int32), ("n_threads", ctypes.c_int32),
        ("softmax_scale", ctypes.c_double),
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

    def _c(self) -> _Params:
        return _Params(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.rank,
                       self.ctx_len, self.group_size, self.n_select, self.kv_dtype,
                       self.meta_dtype, self.reduce, self.head_mode, self.n_threads,
                       self.softmax_scale)

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
        _lib.oracle_dense_attn.argtypes = [pp, vp, vp, vp, vp]
        _lib.oracle_round_to_bf16.argtypes = [ctypes.c_double]
        _lib.oracle_round_to_bf16.restype = ctypes.c_uint16
        for f in (_lib.oracle_build_metadata, _lib.oracle_predict_select,
                  _lib.oracle_sparse_attn, _lib.oracle_dense_attn):
            f.restype = ctypes.c_int
    return _lib


def _np_dtype(code: int):
    return np.float32 if code == F32 else np.uint16


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
    K = _arr(K, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_kv_heads, sh.ctx_len, sh.head_dim), "K")
    A = _arr(A, np.float32, (sh.n_kv_heads, sh.head_dim, sh.rank), "A")
    out = np.empty(sh.sets + (sh.ctx_len, sh.rank), dtype=_np_dtype(sh.meta_dtype))
    exact = np.empty(out.shape, dtype=np.float64) if want_exact else None
    c = sh._c()
    _check(lib().oracle_build_metadata(ctypes.byref(c), _ptr(K), _ptr(A), _ptr(out), _ptr(exact)),
           "oracle_build_metadata")
    return (out, exact) if want_exact else out


def predict_select(sh: Shape, q, K_lr, A):
    """Returns dict(idx [B,H_kv,M] int32 ascending, gs [B,H_kv,NG] f64,
    s [B,H_kv,N] f64, boundary [B,H_kv,2] f64); no H_kv axis in joint mode."""
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    K_lr = _arr(K_lr, _np_dtype(sh.meta_dtype), sh.sets + (sh.ctx_len, sh.rank), "K_lr")
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


def sparse_attn(sh: Shape, q, K, V, idx):
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    shape_kv = (sh.batch, sh.n_kv_heads, sh.ctx_len, sh.head_dim)
    K = _arr(K, _np_dtype(sh.kv_dtype), shape_kv, "K")
    V = _arr(V, _np_dtype(sh.kv_dtype), shape_kv, "V")
    idx = _arr(idx, np.int32, sh.sets + (sh.n_select,), "idx")
    out = np.empty((sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    c = sh._c()
    _check(lib().oracle_sparse_attn(ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(idx), _ptr(out)),
           "oracle_sparse_attn")
    return out


def dense_attn(sh: Shape, q, K, V):
    q = _arr(q, _np_dtype(sh.kv_dtype), (sh.batch, sh.n_q_heads, sh.head_dim), "q")
    shape_kv = (sh.batch, sh.n_kv_heads, sh.ctx_len, sh.head_dim)
    K = _arr(K, _np_dtype(sh.kv_dtype), shape_kv, "K")
    V = _arr(V, _np_dtype(sh.kv_dtype), shape_kv, "V")
    out = np.empty((sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    c = sh._c()
    _check(lib().oracle_dense_attn(ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(out)),
           "oracle_dense_attn")
    return out


def round_to_bf16(x: float) -> int:
    return int(lib().oracle_round_to_bf16(float(x)))
