"""Glue for the GPU parity tests: moves seeded inputs to the device, calls the HIP
path through the C-ABI binding, calls the CPU oracle on the same host arrays, and
implements the comparison rules (index margin rule, attention error metric)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2511_11907_amd as kv
from workloads import Config, LayerInputs, make_layer, storage_to_f32

DEV = "cuda:0"

ATTN_TOL = {"f32": 1e-5, "bf16": 2e-2}   # max |o_gpu - o_ref| / max |o_ref| per (b, h) vector
GS_TOL = 2e-5                            # fp32 accumulation over r <= 128 terms and <= 8 heads
MARGIN = 1e-4                            # relative margin of the index rule


def dt_code(name: str) -> int:
    return {"f32": kv.KVS_F32, "bf16": kv.KVS_BF16, "fp8": kv.KVS_FP8_E4M3}[name]


_FP8_VALUES = np.array([oracle.fp8_e4m3_value(c) for c in range(256)])


def meta_values(x: np.ndarray) -> np.ndarray:
    """Stored metadata (float32, uint16 bf16 bits or uint8 E4M3 codes) -> fp64 values."""
    if x.dtype == np.uint8:
        return _FP8_VALUES[x]
    return storage_to_f32(x).astype(np.float64)


def to_dev(x: np.ndarray) -> torch.Tensor:
    """Storage array (float32, uint16 bf16 bits, int32) -> device tensor."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    if x.dtype == np.uint8:
        return torch.from_numpy(np.ascontiguousarray(x)).to(DEV).view(torch.float8_e4m3fn)
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def to_host_storage(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).cpu().numpy()
    return t.cpu().numpy()


def kv_params(cfg: Config, **over) -> kv.Params:
    d = dict(batch=cfg.batch, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
             head_dim=cfg.head_dim, rank=cfg.rank, ctx_len=cfg.ctx_len,
             group_size=cfg.group_size, n_select=cfg.n_select,
             kv_dtype=dt_code(cfg.dtype), meta_dtype=dt_code(cfg.dtype),
             head_mode=kv.KVS_HEADS_JOINT if cfg.joint else kv.KVS_HEADS_SEPARATE)
    d.update(over)
    if isinstance(d["meta_dtype"], str):
        d["meta_dtype"] = dt_code(d["meta_dtype"])
    return kv.Params(**d)


def orc_shape(cfg: Config, n_threads: int = 8, **over) -> oracle.Shape:
    code = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
    d = dict(batch=cfg.batch, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
             head_dim=cfg.head_dim, rank=cfg.rank, ctx_len=cfg.ctx_len,
             group_size=cfg.group_size, n_select=cfg.n_select, kv_dtype=code, meta_dtype=code,
             n_threads=n_threads,
             head_mode=oracle.HEADS_JOINT if cfg.joint else oracle.HEADS_SEPARATE)
    d.update(over)
    if isinstance(d["meta_dtype"], str):
        d["meta_dtype"] = {"f32": oracle.F32, "bf16": oracle.BF16, "fp8": oracle.FP8_E4M3}[d["meta_dtype"]]
    return oracle.Shape(**d)


def workspace(p: kv.Params) -> torch.Tensor:
    n = kv.kvs_workspace_bytes(p)
    assert n > 0
    # poison everything, then let the library prepare its arrival counters: a kernel that
    # relies on any other part of the scratch being zero shows up as NaN
    ws = torch.full((n // 4,), float("nan"), dtype=torch.float32, device=DEV)
    kv.kvs_workspace_init(p, ws)
    return ws


class DeviceLayer:
    """Device copies of one layer's inputs."""

    def __init__(self, L: LayerInputs):
        self.K, self.V, self.q, self.A = to_dev(L.K), to_dev(L.V), to_dev(L.q), to_dev(L.A)


# ---- comparison rules ---------------------------------------------------------------
def check_index_margin(idx_gpu: np.ndarray, gs_ref: np.ndarray, boundary: np.ndarray, what=""):
    """idx_gpu [M] of one problem against the oracle's scores gs_ref [NG].
    Every group scoring above (M+1)-th + eps must be selected, every group scoring below
    M-th - eps must not; inside the band either is accepted.  The set must hold M unique,
    in-range, ascending indices.  Returns True if the comparison was bit-exact set
    equality (margin wider than the band)."""
    M, NG = idx_gpu.shape[0], gs_ref.shape[0]
    assert idx_gpu.min() >= 0 and idx_gpu.max() < NG, what
    assert np.all(np.diff(idx_gpu) > 0), f"{what}: idx not strictly ascending"
    t_hi, t_lo = boundary
    if not np.isfinite(t_lo):      # M == NG: everything is selected
        np.testing.assert_array_equal(idx_gpu, np.arange(NG))
        return True
    eps = MARGIN * max(abs(t_hi), abs(t_lo), 1e-3 * np.abs(gs_ref).max())
    sel = np.zeros(NG, bool)
    sel[idx_gpu] = True
    must = gs_ref > t_lo + eps
    must_not = gs_ref < t_hi - eps
    assert not np.any(must & ~sel), f"{what}: {int((must & ~sel).sum())} clear winners missing"
    assert not np.any(must_not & sel), f"{what}: {int((must_not & sel).sum())} clear losers selected"
    return (t_hi - t_lo) > eps


def attn_error(out_gpu: np.ndarray, out_ref: np.ndarray) -> float:
    """max over (b, h) of  max_i |gpu - ref| / max_i |ref|."""
    g = out_gpu.astype(np.float64).reshape(-1, out_gpu.shape[-1])
    r = out_ref.reshape(-1, out_ref.shape[-1])
    return float((np.abs(g - r).max(1) / np.abs(r).max(1)).max())


def out_values(t: torch.Tensor) -> np.ndarray:
    return storage_to_f32(to_host_storage(t)).astype(np.float64)


# ---- one full comparison of a small configuration --------------------------------------
def run_and_compare(cfg: Config, reduce: int = 0, layer: int = 0, check_meta: bool = True,
                    meta: str = None, meta_scale: float = 0.0, meta_scales: np.ndarray = None):
    """Whole path at a size the oracle finishes in seconds: metadata, prediction and
    selection, attention with the oracle's indices, and the fused decode step.
    `meta` overrides the metadata dtype ("f32", "bf16", "fp8"); `meta_scales` (one per
    selection set) overrides `meta_scale`."""
    L = make_layer(cfg, layer)
    D = DeviceLayer(L)
    meta = meta or cfg.dtype
    p = kv_params(cfg, reduce=reduce, meta_dtype=meta, meta_scale=meta_scale)
    sh = orc_shape(cfg, reduce=reduce, meta_dtype=meta, meta_scale=meta_scale)
    if meta_scales is not None:
        p.meta_scales = torch.from_numpy(np.ascontiguousarray(meta_scales, dtype=np.float32)).to(DEV)
        # (the oracle gets exactly the fp32 values the library reads)
        sh = orc_shape(cfg, reduce=reduce, meta_dtype=meta,
                       meta_scales=np.ascontiguousarray(meta_scales, dtype=np.float32).astype(np.float64))
    B, Hk, N, r, M = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.rank, cfg.n_select
    stats = {}

    # metadata: oracle-rounded K_lr is the reference and the input of the next step
    klr_ref, klr_exact = oracle.build_metadata(sh, L.K, L.A, want_exact=True)
    if check_meta:
        klr_gpu = torch.empty(p.sets + (N, r), dtype=to_dev(klr_ref[..., :1, :]).dtype, device=DEV)
        kv.kvs_build_metadata(p, D.K, D.A, klr_gpu)
        torch.cuda.synchronize()
        # joint-head mode contracts over the H_kv*d flattened key row
        absdot = np.einsum("bknd,kdr->bnr" if cfg.joint else "bknd,kdr->bknr",
                           np.abs(storage_to_f32(L.K)).astype(np.float64), np.abs(L.A).astype(np.float64))
        terms = cfg.head_dim * (Hk if cfg.joint else 1)
        sc = meta_scale or 1.0        # stored units: K.A / meta_scale
        if meta_scales is not None:
            sc = np.ascontiguousarray(meta_scales, dtype=np.float32).astype(np.float64)[..., None, None]
        stats["meta_mismatch"] = compare_metadata(to_host_storage(klr_gpu), klr_ref, klr_exact / sc,
                                                  absdot / sc, terms, meta)

    ws = workspace(p)
    klr_dev = to_dev(klr_ref)
    ref = oracle.predict_select(sh, L.q, klr_ref, L.A)
    idx = torch.full(p.sets + (M,), -1, dtype=torch.int32, device=DEV)
    gs = torch.full(p.sets + (cfg.n_groups,), float("nan"), dtype=torch.float32, device=DEV)
    kv.kvs_predict_select(p, D.q, klr_dev, D.A, idx, gs, ws)
    torch.cuda.synchronize()
    gs_h, idx_h = gs.cpu().numpy().astype(np.float64), idx.cpu().numpy()
    scale = np.abs(ref["gs"]).max()
    stats["gs_err"] = float(np.abs(gs_h - ref["gs"]).max() / scale)
    assert stats["gs_err"] <= GS_TOL, stats
    exact = 0
    flat = lambda a: a.reshape((-1,) + a.shape[len(p.sets):])   # one row per selection set
    for i, (ig, gr, bd, ir) in enumerate(zip(flat(idx_h), flat(ref["gs"]), flat(ref["boundary"]),
                                             flat(ref["idx"]))):
        exact += check_index_margin(ig, gr, bd, f"{cfg.name} set {i}")
        if (bd[0] - bd[1]) > MARGIN * scale:
            np.testing.assert_array_equal(ig, ir)
    stats["idx_exact_problems"] = int(exact)

    # attention on the oracle's indices
    out_ref = oracle.sparse_attn(sh, L.q, L.K, L.V, ref["idx"])
    out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=D.q.dtype, device=DEV)
    kv.kvs_sparse_decode_attn(p, D.q, D.K, D.V, to_dev(ref["idx"]), out, ws)
    torch.cuda.synchronize()
    stats["attn_err"] = attn_error(out_values(out), out_ref)
    assert stats["attn_err"] <= ATTN_TOL[cfg.dtype], stats

    # whole step in one call; attention is compared on the indices the GPU chose
    idx2 = torch.full_like(idx, -1)
    out2 = torch.full_like(out, float("nan"))
    kv.kvs_decode_step(p, D.q, klr_dev, D.A, D.K, D.V, idx2, None, out2, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx2.cpu().numpy(), idx_h)
    out_ref2 = out_ref if np.array_equal(idx_h, ref["idx"]) else oracle.sparse_attn(sh, L.q, L.K, L.V, idx_h)
    stats["step_err"] = attn_error(out_values(out2), out_ref2)
    assert stats["step_err"] <= ATTN_TOL[cfg.dtype], stats
    return stats


# ---- full-size configurations, oracle on sampled problems ------------------------------------
def full_size_sampled(cfg: Config, samples, budgets=None, layer=0, meta: str = None,
                      meta_scale: float = 0.0):
    """GPU on the whole batch at the real size; oracle on the sampled (b, k) problems.
    The metadata of the sampled problems is built by the oracle and written over the
    GPU-built rows, so both sides score exactly the same K_lr."""
    L = make_layer(cfg, layer, workers=16)
    D = DeviceLayer(L)
    meta = meta or cfg.dtype
    mk = dict(meta_dtype=meta, meta_scale=meta_scale)
    sc = meta_scale or 1.0
    p = kv_params(cfg, **mk)
    B, Hk, N, r, qpk = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.rank, cfg.q_per_kv
    klr = torch.empty((B, Hk, N, r), dtype=kv.binding._dtype_of(p.meta_dtype), device=DEV)
    kv.kvs_build_metadata(p, D.K, D.A, klr)
    torch.cuda.synchronize()
    sub = {}
    for (b, k) in samples:
        sh1 = orc_shape(cfg, batch=1, n_kv_heads=1, n_q_heads=qpk, **mk)
        K1, V1 = L.K[b:b + 1, k:k + 1], L.V[b:b + 1, k:k + 1]
        q1, A1 = L.q[b:b + 1, k * qpk:(k + 1) * qpk], L.A[k:k + 1]
        klr1, exact1 = oracle.build_metadata(sh1, K1, A1, want_exact=True)
        absdot = np.abs(storage_to_f32(K1)).astype(np.float64)[0, 0] @ np.abs(A1[0]).astype(np.float64)
        frac = compare_metadata(to_host_storage(klr[b, k]), klr1[0, 0], exact1[0, 0] / sc, absdot / sc,
                                cfg.head_dim, meta)
        klr[b, k].copy_(to_dev(klr1[0, 0]))
        sub[(b, k)] = (sh1, K1, V1, q1, A1, klr1, frac)
    results = {}
    for M in (budgets or [cfg.n_select]):
        pM = kv_params(cfg, n_select=M, **mk)
        ws = workspace(pM)
        idx = torch.full((B, Hk, M), -1, dtype=torch.int32, device=DEV)
        out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=D.q.dtype, device=DEV)
        kv.kvs_decode_step(pM, D.q, klr, D.A, D.K, D.V, idx, None, out, ws)
        torch.cuda.synchronize()
        idx_h, out_h = idx.cpu().numpy(), out_values(out)
        # properties that hold for every problem at any size
        assert np.all(np.diff(idx_h, axis=-1) > 0) and idx_h.min() >= 0 and idx_h.max() < cfg.n_groups
        assert np.isfinite(out_h).all()
        worst = 0.0
        for (b, k), (sh1, K1, V1, q1, A1, klr1, frac) in sub.items():
            shM = orc_shape(cfg, batch=1, n_kv_heads=1, n_q_heads=qpk, n_select=M, **mk)
            ref = oracle.predict_select(shM, q1, klr1, A1)
            check_index_margin(idx_h[b, k], ref["gs"][0, 0], ref["boundary"][0, 0], f"{cfg.name} M={M} b={b} k={k}")
            out_ref = oracle.sparse_attn(shM, q1, K1, V1, idx_h[b:b + 1, k:k + 1])
            err = attn_error(out_h[b:b + 1, k * qpk:(k + 1) * qpk], out_ref)
            assert err <= ATTN_TOL[cfg.dtype], (cfg.name, M, b, k, err)
            if M == cfg.n_groups:   # 100 % budget: the step is dense attention
                dense = oracle.dense_attn(shM, q1, K1, V1)
                assert attn_error(out_h[b:b + 1, k * qpk:(k + 1) * qpk], dense) <= ATTN_TOL[cfg.dtype]
            worst = max(worst, err)
        results[M] = worst
    print(f"[parity] {cfg.name}_full meta={meta}: " + ", ".join(f"M={m}: {e:.3g}" for m, e in results.items()),
          flush=True)
    return results



def full_size_all(cfg: Config, layer=0, threads: int = 16):
    """GPU on the whole batch at the real size, oracle on EVERY (b, k) problem (its own
    threading over the independent problems).  The oracle's metadata is what both sides
    score.  Returns (problems, problems compared by exact set equality, worst attention
    error)."""
    import time
    t0 = time.time()
    L = make_layer(cfg, layer, workers=16)
    D = DeviceLayer(L)
    p = kv_params(cfg)
    sh = orc_shape(cfg, n_threads=threads)
    B, Hk, N, r = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.rank
    klr_gpu = torch.empty((B, Hk, N, r), dtype=kv.binding._dtype_of(p.meta_dtype), device=DEV)
    kv.kvs_build_metadata(p, D.K, D.A, klr_gpu)
    torch.cuda.synchronize()
    klr_ref, klr_exact = oracle.build_metadata(sh, L.K, L.A, want_exact=True)
    klr_gpu_h = to_host_storage(klr_gpu)
    worst_frac = 0.0
    for b in range(B):
        for k in range(Hk):
            absdot = np.abs(storage_to_f32(L.K[b, k])).astype(np.float64) @ np.abs(L.A[k]).astype(np.float64)
            worst_frac = max(worst_frac, compare_metadata(klr_gpu_h[b, k], klr_ref[b, k], klr_exact[b, k],
                                                          absdot, cfg.head_dim, cfg.dtype))
    del klr_exact, klr_gpu_h
    ws = workspace(p)
    idx = torch.full((B, Hk, cfg.n_select), -1, dtype=torch.int32, device=DEV)
    out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=D.q.dtype, device=DEV)
    kv.kvs_decode_step(p, D.q, to_dev(klr_ref), D.A, D.K, D.V, idx, None, out, ws)
    torch.cuda.synchronize()
    idx_h, out_h = idx.cpu().numpy(), out_values(out)
    ref = oracle.predict_select(sh, L.q, klr_ref, L.A)
    exact = 0
    for b in range(B):
        for k in range(Hk):
            if check_index_margin(idx_h[b, k], ref["gs"][b, k], ref["boundary"][b, k], f"{cfg.name} b={b} k={k}"):
                np.testing.assert_array_equal(idx_h[b, k], ref["idx"][b, k])
                exact += 1
    out_ref = oracle.sparse_attn(sh, L.q, L.K, L.V, idx_h)
    err = attn_error(out_h, out_ref)
    assert err <= ATTN_TOL[cfg.dtype], (cfg.name, err)
    print(f"[parity] {cfg.name}_full_all: {B * Hk} problems, {exact} by exact set equality, "
          f"attention err {err:.3g}, metadata mismatch <= {worst_frac:.2g}, {time.time() - t0:.1f} s", flush=True)
    return B * Hk, exact, err


def _ulp(v: np.ndarray, dtype: str) -> np.ndarray:
    """Spacing of the storage dtype at |v| (normal range; E4M3 also below it)."""
    if dtype == "f32":
        return np.spacing(np.abs(v).astype(np.float32)).astype(np.float64)
    if dtype == "fp8":
        e = np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -6)))
        return 2.0 ** (e - 3)
    e = np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126)))
    return 2.0 ** (e - 7)


def compare_metadata(klr_gpu: np.ndarray, klr_ref: np.ndarray, klr_exact: np.ndarray,
                     absdot: np.ndarray, d: int, dtype: str) -> float:
    """GPU K_lr (fp32 accumulation over d terms, one rounding) against the oracle's exact
    fp64 products: every element must lie within half a unit in the last place of the
    storage dtype plus the fp32 accumulation bound d * 2^-24 * sum_i |K_i A_ij|.  For bf16
    and fp8 storage the result must also be bit-identical to the oracle's rounding except
    where the exact value sits that close to a rounding boundary (a fraction of a per cent
    of the well-conditioned elements).  Returns that fraction."""
    g = meta_values(klr_gpu)
    r = meta_values(klr_ref)
    if dtype == "fp8":     # saturating format: compare against the clamped exact value
        klr_exact = np.clip(klr_exact, -448.0, 448.0)
    acc = (d + 2) * 2.0 ** -24 * absdot      # fp32 accumulation, plus the division by the scale
    ulp = np.maximum(_ulp(g, dtype), _ulp(klr_exact, dtype))
    assert np.all(np.abs(g - klr_exact) <= 0.5 * ulp + acc + 1e-300), \
        "GPU metadata is further from the exact product than rounding + fp32 accumulation allow"
    # Bit-identity with the oracle's rounding is asked only of well-conditioned elements:
    # where the products cancel to far below their magnitudes (an adapter column orthogonal
    # to every key of a short context) the fp32 accumulation error exceeds the spacing of
    # the narrow dtype at the tiny result, and only the bound above can hold.
    well = np.abs(klr_exact) > 1024.0 * acc
    frac = float((g != r)[well].mean()) if well.any() else 0.0
    if dtype in ("bf16", "fp8"):
        assert frac <= 2e-3, f"too many metadata elements differ from the oracle: {frac}"
    return frac
