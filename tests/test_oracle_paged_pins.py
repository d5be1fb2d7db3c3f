"""Pins of the oracle's mapping-table attention (Sec. 3.4.4 "KV cache manager": KV groups
are addressed logically, a table says where they physically are) and of the selection
overlap count (Sec. 3.4.2: overlap ratio of consecutive steps), against things other
than itself."""
import numpy as np
import pytest

import oracle
from oracle import Shape
import brute


def _problem(seed, B=2, Hq=4, Hk=2, d=8, N=32):
    g = np.random.default_rng(seed)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    V = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    return K, V, q


def _rand_idx(seed, lead, NG, M):
    g = np.random.default_rng(seed)
    n = int(np.prod(lead))
    return np.stack([np.sort(g.choice(NG, M, replace=False)) for _ in range(n)]).astype(np.int32).reshape(lead + (M,))


def _as_pool(K, G):
    """Cache [B,H,N,d] viewed as slots [B*H*NG, G, d] with the identity table."""
    B, Hk, N, d = K.shape
    NG = N // G
    pool = np.ascontiguousarray(K.reshape(B * Hk * NG, G, d))
    table = np.arange(B * Hk * NG, dtype=np.int32).reshape(B, Hk, NG)
    return pool, table


@pytest.mark.parametrize("joint", [False, True])
def test_identity_table_over_the_cache_equals_the_unpaged_call(joint):
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 32, 4, 3
    K, V, q = _problem(1)
    sh = Shape(B, Hq, Hk, d, 4, N, G, M, head_mode=oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE)
    idx = _rand_idx(2, sh.sets, N // G, M)
    Kp, table = _as_pool(K, G)
    Vp, _ = _as_pool(V, G)
    np.testing.assert_array_equal(oracle.sparse_attn_paged(sh, q, Kp, Vp, table, idx),
                                  oracle.sparse_attn(sh, q, K, V, idx))


def test_shuffled_slots_with_spare_poisoned_slots_give_the_same_output():
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 32, 4, 3
    K, V, q = _problem(3)
    sh = Shape(B, Hq, Hk, d, 4, N, G, M)
    idx = _rand_idx(4, sh.sets, N // G, M)
    Kp, table = _as_pool(K, G)
    Vp, _ = _as_pool(V, G)
    g = np.random.default_rng(5)
    n_used, n_slots = Kp.shape[0], Kp.shape[0] + 7
    where = g.permutation(n_slots)[:n_used].astype(np.int32)      # new slot of each old slot
    K2 = np.full((n_slots, G, d), np.nan, np.float32)
    V2 = np.full((n_slots, G, d), np.nan, np.float32)
    K2[where], V2[where] = Kp, Vp
    table2 = where[table]
    rbK = g.standard_normal((B, Hk, 5, d)).astype(np.float32)
    rbV = g.standard_normal((B, Hk, 5, d)).astype(np.float32)
    np.testing.assert_array_equal(oracle.sparse_attn_paged(sh, q, K2, V2, table2, idx, rbK, rbV, 3),
                                  oracle.sparse_attn(sh, q, K, V, idx, rbK, rbV, 3))


def test_paged_attention_matches_brute_force_over_the_gathered_rows():
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 24, 4, 2
    NG = N // G
    g = np.random.default_rng(6)
    n_slots = 40
    Kp = g.standard_normal((n_slots, G, d)).astype(np.float32)
    Vp = g.standard_normal((n_slots, G, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    table = g.integers(0, n_slots, (B, Hk, NG)).astype(np.int32)   # slots may even be shared
    idx = _rand_idx(7, (B, Hk), NG, M)
    sh = Shape(B, Hq, Hk, d, 4, N, G, M)
    out = oracle.sparse_attn_paged(sh, q, Kp, Vp, table, idx)
    # gather by hand into a dense per-problem cache and use the dense softmax routine
    Kd = np.zeros((B, Hk, M * G, d)); Vd = np.zeros((B, Hk, M * G, d))
    for b in range(B):
        for k in range(Hk):
            slots = table[b, k, idx[b, k]]
            Kd[b, k] = Kp[slots].reshape(M * G, d)
            Vd[b, k] = Vp[slots].reshape(M * G, d)
    np.testing.assert_allclose(out, brute.dense_attention(q.astype(np.float64), Kd, Vd), rtol=1e-12, atol=1e-13)


def test_slot_outside_the_pool_is_rejected():
    K, V, q = _problem(8)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    idx = _rand_idx(1, sh.sets, 8, 3)
    Kp, table = _as_pool(K, 4)
    Vp, _ = _as_pool(V, 4)
    bad = table.copy()
    bad[0, 0, idx[0, 0, 0]] = Kp.shape[0]
    with pytest.raises(RuntimeError):
        oracle.sparse_attn_paged(sh, q, Kp, Vp, bad, idx)


@pytest.mark.parametrize("joint", [False, True])
def test_overlap_count_matches_set_intersection(joint):
    B, Hk, NG, M = 3, 2, 64, 17
    sh = Shape(B, 4, Hk, 8, 4, NG * 4, 4, M, head_mode=oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE)
    a, b = _rand_idx(1, sh.sets, NG, M), _rand_idx(2, sh.sets, NG, M)
    got = oracle.selection_overlap(sh, a, b)
    want = np.array([len(np.intersect1d(x, y)) for x, y in zip(a.reshape(-1, M), b.reshape(-1, M))],
                    dtype=np.int32).reshape(sh.sets)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(oracle.selection_overlap(sh, a, a), np.full(sh.sets, M, np.int32))
    # order does not matter; disjoint selections share nothing
    np.testing.assert_array_equal(oracle.selection_overlap(sh, a[..., ::-1].copy(), b), want)
    lo = np.tile(np.arange(M, dtype=np.int32), sh.sets + (1,))
    np.testing.assert_array_equal(oracle.selection_overlap(sh, lo, lo + M), np.zeros(sh.sets, np.int32))
