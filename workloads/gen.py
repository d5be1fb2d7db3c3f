"""Deterministic synthetic decode-step inputs.

Every tensor is drawn from a counter-based generator (numpy Philox) keyed by
(seed, layer, sequence, kv head, tensor id), so any single (sequence, kv head)
problem can be regenerated alone, on any machine, without generating the rest.

The recipe mirrors the premise of the method (Sec. 3.2-4.3 of the paper): keys
of one KV head live close to a low-dimensional subspace (so a rank-r adapter
captures them), and a small set of tokens dominates the scores.

    basis  Bm[l,k]   : rho x d,  N(0,1)/sqrt(rho)        (shared by all sequences)
    K[l,s,k]         : Z @ Bm + noise_std * N(0,1),  Z : N x rho ~ N(0,1)
                       heavy-hitter rows multiplied by heavy_scale
    V[l,s,k]         : N(0,1)
    q[l,s,h]         : N(0,1)
    A[l,k]           : top-r right singular vectors of sequence 0's K[l,0,k]
                       (the offline adapter of Sec. 3.2, fitted on a
                       "calibration" sequence and reused for the whole batch)

Values are cast to the config's storage dtype (fp32, or bf16 with
round-to-nearest-even).  Nothing here belongs to the decode step itself.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional

import numpy as np

# tensor ids entering the generator key
_T_BASIS, _T_Z, _T_NOISE, _T_HEAVY, _T_V, _T_Q = 1, 2, 3, 4, 5, 6
_SEQ_SHARED = 0xFFFF  # "sequence" slot of tensors shared by the whole batch
_HEAD_SHARED = 0xFFFF  # "head" slot of draws shared by all KV heads (joint-head workloads)


@dataclass(frozen=True)
class Config:
    name: str
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_len: int
    rank: int
    group_size: int
    n_select: int
    dtype: str            # "f32" or "bf16": storage type of K, V, q, out and K_lr
    planted_rank: int     # rho
    noise_std: float
    heavy: float          # >= 1: heavy-hitter tokens per (sequence, kv head); < 1: fraction of tokens
    heavy_scale: float = 4.0
    seed: int = 0
    joint: bool = False   # joint-head design: one adapter over the flattened keys of all KV heads

    @property
    def n_groups(self) -> int:
        return self.ctx_len // self.group_size

    @property
    def q_per_kv(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)

    def n_heavy(self) -> int:
        if self.heavy >= 1:
            return int(self.heavy)
        return int(math.ceil(self.heavy * self.ctx_len)) if self.heavy > 0 else 0


def budget_to_groups(budget: float, n_groups: int) -> int:
    """Number of selected groups for a fractional budget: ceil(budget * NG).

    10 % of 8192 groups is 819.2 and the workload table fixes 820, hence ceil.
    The product is formed in exact integer arithmetic on the per-mille grid so
    that e.g. 0.05 * 4096 = 204.8 cannot round the wrong way.
    """
    ppm = int(round(budget * 1_000_000))
    m = -((-ppm * n_groups) // 1_000_000)
    return max(1, min(n_groups, m))


PRESETS = {
    # single layer, 8q/2kv, d=64, 4K context, fp32, r=16, G=4, 64 groups per kv head
    "c1": Config("c1", 1, 1, 8, 2, 64, 4096, 16, 4, 64, "f32", 16, 0.1, 0),
    # 4B-class GQA layer, b=1, 32q/8kv, d=128, 32K, bf16, r=32, G=4, 10 % of 8192 groups
    "c2": Config("c2", 1, 1, 32, 8, 128, 32768, 32, 4, 820, "bf16", 32, 0.1, 16),
    # same layer, b=8, independent seeds per sequence
    "c3": Config("c3", 1, 8, 32, 8, 128, 32768, 32, 4, 820, "bf16", 32, 0.1, 16),
    # 8B-class long context, b=4, 128K, r=64, G=8, 2048 groups, 1 % heavy hitters
    "c4": Config("c4", 1, 4, 32, 8, 128, 131072, 64, 8, 2048, "bf16", 64, 0.1, 0.01),
    # 36-layer stack, b=16, 16K, r=32, G=4, 5 % of 4096 groups
    "c5": Config("c5", 36, 16, 32, 8, 128, 16384, 32, 4, 205, "bf16", 32, 0.1, 16),
}
# the same workloads under the joint-head design (compression ratio H_kv*d/r = 32, 32, 16, 32)
PRESETS.update({k + "j": v.replace(name=k + "j", joint=True) for k, v in list(PRESETS.items())})


# --------------------------------------------------------------------------
# dtype casts
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even, finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    """Cast to the storage form: float32 array, or uint16 bf16 bit patterns."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f32(x: np.ndarray) -> np.ndarray:
    """Storage form -> fp32 values (exact for both dtypes)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x)
    return np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _rng(cfg: Config, layer: int, seq: int, head: int, tensor: int) -> np.random.Generator:
    key = (
        (int(cfg.seed) & 0xFFFFFFFF)
        | (int(layer) & 0xFFFF) << 32
        | (int(seq) & 0xFFFF) << 48
        | (int(head) & 0xFFFF) << 64
        | (int(tensor) & 0xFF) << 80
    )
    return np.random.Generator(np.random.Philox(key=key))


def _basis(cfg: Config, layer: int, kv_head: int) -> np.ndarray:
    g = _rng(cfg, layer, _SEQ_SHARED, kv_head, _T_BASIS)
    b = g.standard_normal((cfg.planted_rank, cfg.head_dim), dtype=np.float32)
    return b / np.float32(math.sqrt(cfg.planted_rank))


def make_problem_kv(cfg: Config, layer: int, seq: int, kv_head: int):
    """K and V of one (layer, sequence, kv head): storage arrays of shape [N, d]."""
    n, d = cfg.ctx_len, cfg.head_dim
    # joint-head workloads: the latent factors (and the heavy-hitter tokens) of a token are
    # shared by all KV heads, so the flattened row [K_0 | ... | K_{H-1}] has the planted rank
    # and one adapter over it can capture what rho columns capture per head
    zh = _HEAD_SHARED if cfg.joint else kv_head
    z = _rng(cfg, layer, seq, zh, _T_Z).standard_normal((n, cfg.planted_rank), dtype=np.float32)
    k = z @ _basis(cfg, layer, kv_head)
    del z
    if cfg.noise_std:
        noise = _rng(cfg, layer, seq, kv_head, _T_NOISE).standard_normal((n, d), dtype=np.float32)
        noise *= np.float32(cfg.noise_std)
        k += noise
        del noise
    nh = cfg.n_heavy()
    if nh:
        rows = _rng(cfg, layer, seq, zh, _T_HEAVY).choice(n, size=min(nh, n), replace=False)
        k[rows] *= np.float32(cfg.heavy_scale)
    v = _rng(cfg, layer, seq, kv_head, _T_V).standard_normal((n, d), dtype=np.float32)
    return _store(k, cfg.dtype), _store(v, cfg.dtype)


def make_q(cfg: Config, layer: int, seq: int) -> np.ndarray:
    """Query vectors of one (layer, sequence): storage array [H_q, d]."""
    q = _rng(cfg, layer, seq, 0, _T_Q).standard_normal((cfg.n_q_heads, cfg.head_dim), dtype=np.float32)
    return _store(q, cfg.dtype)


def fit_adapter(k_calib: np.ndarray, rank: int) -> np.ndarray:
    """Offline low-rank adapter (Sec. 3.2): top-`rank` right singular vectors of
    the calibration keys [N, d], as an fp32 [d, rank] matrix with orthonormal
    columns, ordered by decreasing singular value.  Computed from the
    eigen-decomposition of the d x d Gram matrix in fp64; each column's sign is
    fixed so that its largest-magnitude entry is positive."""
    kc = storage_to_f32(k_calib).astype(np.float64)
    gram = kc.T @ kc
    w, vecs = np.linalg.eigh(gram)
    order = np.argsort(w)[::-1][:rank]
    a = vecs[:, order]
    piv = np.argmax(np.abs(a), axis=0)
    sign = np.sign(a[piv, np.arange(a.shape[1])])
    sign[sign == 0] = 1.0
    return np.ascontiguousarray((a * sign).astype(np.float32))


@dataclass
class LayerInputs:
    cfg: Config
    layer: int
    K: np.ndarray   # [B, H_kv, N, d] storage (float32 or uint16 bf16 bits)
    V: np.ndarray   # [B, H_kv, N, d]
    q: np.ndarray   # [B, H_q, d]
    A: np.ndarray   # [H_kv, d, r] float32 (joint-head: the [(H_kv d), r] adapter, same layout)


def make_layer(cfg: Config, layer: int = 0, workers: int = 8,
               seq_offset: int = 0, adapter_from: Optional[np.ndarray] = None) -> LayerInputs:
    """All inputs of one layer.  `seq_offset` shifts the sequence ids (used to
    draw several independent copies of a workload); the adapter is always the
    one of sequence 0 of that layer unless `adapter_from` supplies it."""
    b, hk, n, d = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.head_dim
    np_dt = np.float32 if cfg.dtype == "f32" else np.uint16
    K = np.empty((b, hk, n, d), dtype=np_dt)
    V = np.empty((b, hk, n, d), dtype=np_dt)

    def job(sk):
        s, k = sk
        K[s, k], V[s, k] = make_problem_kv(cfg, layer, seq_offset + s, k)

    jobs = [(s, k) for s in range(b) for k in range(hk)]
    if workers > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(job, jobs))
    else:
        for j in jobs:
            job(j)

    q = np.stack([make_q(cfg, layer, seq_offset + s) for s in range(b)])
    if adapter_from is not None:
        A = np.ascontiguousarray(adapter_from, dtype=np.float32)
    elif cfg.joint:
        k0 = [K[0, k] if seq_offset == 0 else make_problem_kv(cfg, layer, 0, k)[0] for k in range(hk)]
        flat = np.concatenate([storage_to_f32(x) for x in k0], axis=1)      # [N, H_kv*d], head-major
        A = fit_adapter(flat, cfg.rank).reshape(hk, d, cfg.rank)
    else:
        A = np.empty((hk, d, cfg.rank), dtype=np.float32)
        for k in range(hk):
            if seq_offset == 0:
                k0 = K[0, k]
            else:
                k0, _ = make_problem_kv(cfg, layer, 0, k)
            A[k] = fit_adapter(k0, cfg.rank)
    return LayerInputs(cfg, layer, K, V, q, A)
