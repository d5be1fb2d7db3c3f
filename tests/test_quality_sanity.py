"""Sanity of the method on the synthetic workloads (not a parity test): on keys that lie
close to a low-dimensional subspace, the low-rank predictor must find most of the groups
that exact q.K scores would pick, and heavy-hitter tokens must be over-represented in the
selection -- the premise of Sec. 3.1-3.3 (few tokens dominate; a compressed K cache is
enough to rank them).  CPU only, through the oracle."""
import numpy as np
import pytest

import oracle
from workloads import PRESETS, make_layer, storage_to_f32


def _exact_group_scores(cfg, L, joint):
    K = storage_to_f32(L.K).astype(np.float64)
    q = storage_to_f32(L.q).astype(np.float64)
    qpk = cfg.q_per_kv
    s = np.einsum("bkhd,bknd->bkn", q.reshape(cfg.batch, cfg.n_kv_heads, qpk, cfg.head_dim), K)
    if joint:
        s = s.sum(axis=1)
    return s.reshape(s.shape[:-1] + (cfg.n_groups, cfg.group_size)).max(-1)


@pytest.mark.parametrize("name", ["c1", "c2", "c2j"])
def test_low_rank_prediction_recalls_the_true_top_groups(name):
    cfg = PRESETS[name].replace(batch=2, ctx_len=4096, n_select=103 if name != "c1" else 64)
    L = make_layer(cfg)
    code = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
    sh = oracle.Shape(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.rank, cfg.ctx_len,
                      cfg.group_size, cfg.n_select, code, code, n_threads=8,
                      head_mode=oracle.HEADS_JOINT if cfg.joint else oracle.HEADS_SEPARATE)
    klr = oracle.build_metadata(sh, L.K, L.A)
    pred = oracle.predict_select(sh, L.q, klr, L.A)["idx"]
    exact = _exact_group_scores(cfg, L, cfg.joint)
    M = cfg.n_select
    truth = np.sort(np.argsort(-exact, axis=-1, kind="stable")[..., :M], axis=-1)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    recall = np.mean([len(np.intersect1d(a, b)) / M for a, b in zip(flat(pred), flat(truth))])
    # sequence 0 is the calibration sample of the adapter; the others share the planted
    # subspace only (as a deployed adapter would), so the bar is the same for all
    assert recall >= 0.9, recall


def test_heavy_hitter_tokens_are_over_represented_in_the_selection():
    cfg = PRESETS["c2"].replace(batch=2, ctx_len=8192, n_select=205)      # 10 % of 2048 groups
    L = make_layer(cfg)
    sh = oracle.Shape(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.rank, cfg.ctx_len,
                      cfg.group_size, cfg.n_select, oracle.BF16, oracle.BF16, n_threads=8)
    klr = oracle.build_metadata(sh, L.K, L.A)
    idx = oracle.predict_select(sh, L.q, klr, L.A)["idx"]
    # heavy hitters = rows whose norm stands out (they were scaled by 4)
    K = storage_to_f32(L.K).astype(np.float64)
    norms = np.linalg.norm(K, axis=-1)                                    # [B, Hk, N]
    hit = 0
    total = 0
    for b in range(cfg.batch):
        for k in range(cfg.n_kv_heads):
            heavy = np.argsort(-norms[b, k])[:cfg.n_heavy()]
            groups = set((heavy // cfg.group_size).tolist())
            hit += len(groups & set(idx[b, k].tolist()))
            total += len(groups)
    # a random 10 % selection would hold 10 % of them; scaled keys score 4x as far from zero, so
    # about half of them land on the selected (positive) side of the ranking
    assert hit / total >= 0.3, hit / total
