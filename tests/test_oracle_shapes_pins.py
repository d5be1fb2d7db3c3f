"""Pins of the CPU oracle at the group sizes and head ratios of the paper's own operating
range, against the independent numpy brute force (no GPU needed).

Group sizes: the parameter solver searches G upwards from 1 in steps of one (App. A.4)
and the appendix's rolling-buffer table reports G = 12, so G is any small integer, not
only a power of two.  Head ratios: the evaluated models (Sec. 4.1) have 3 (LLaMA3-3B),
4 (LLaMA3-8B, Qwen3-4B/8B), 5 (Qwen3-14B, InternVL3-14B), 7 (Qwen2.5-VL-7B) and
8 (Qwen2.5-VL-3B) query heads per KV head.  A slip that only shows off the powers of
two -- a shift where a division belongs, a mask for a remainder, a head loop with a
fixed trip count -- breaks these.
"""
import numpy as np
import pytest

import oracle
from oracle import Shape
import brute


def _problem(seed, B, Hq, Hk, d, r, N):
    g = np.random.default_rng(seed)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    V = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.stack([np.linalg.qr(g.standard_normal((d, r)))[0] for _ in range(Hk)])
    return K, V, q, np.ascontiguousarray(A.astype(np.float32))


def _check(sh, K, V, q, A, mean=False):
    G, M = sh.group_size, sh.n_select
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    s_ref = brute.scores(q.astype(np.float64), klr.astype(np.float64), A.astype(np.float64))
    np.testing.assert_allclose(res["s"], s_ref, rtol=1e-12, atol=1e-13)
    gs_ref = brute.group_scores(s_ref, G, mean=mean)
    np.testing.assert_allclose(res["gs"], gs_ref, rtol=1e-12, atol=1e-13)
    idx_ref = brute.topk_groups(res["gs"], M)
    np.testing.assert_array_equal(res["idx"], idx_ref)
    out = oracle.sparse_attn(sh, q, K, V, res["idx"])
    out_ref = brute.sparse_attention(q.astype(np.float64), K.astype(np.float64),
                                     V.astype(np.float64), idx_ref, G)
    np.testing.assert_allclose(out, out_ref, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mean", [False, True])
@pytest.mark.parametrize("G", [3, 5, 6, 7, 12])
def test_group_sizes_off_the_powers_of_two(G, mean):
    N = 420                      # divisible by 3, 5, 6, 7 and 12
    NG = N // G
    for seed, M in enumerate(sorted({1, NG // 3, NG - 1, NG})):
        K, V, q, A = _problem(100 * G + seed, 2, 4, 2, 8, 4, N)
        sh = Shape(2, 4, 2, 8, 4, N, G, M,
                   reduce=oracle.REDUCE_MEAN if mean else oracle.REDUCE_MAX)
        _check(sh, K, V, q, A, mean)


@pytest.mark.parametrize("Hq,Hk", [(6, 2), (5, 1), (10, 2), (12, 2), (7, 1), (14, 2), (24, 8)])
def test_head_ratios_of_the_evaluated_models(Hq, Hk):
    for seed, (G, M) in enumerate([(4, 5), (3, 7)]):
        K, V, q, A = _problem(7 * Hq + seed, 2, Hq, Hk, 8, 4, 48)
        _check(Shape(2, Hq, Hk, 8, 4, 48, G, M), K, V, q, A)


def test_head_sum_uses_every_head_of_an_odd_ratio():
    """With 5 heads per KV head, zeroing any single query head changes the token scores of
    its own KV head and of no other (a head loop that stops at 4 would miss head 4)."""
    K, V, q, A = _problem(3, 1, 10, 2, 8, 4, 24)
    sh = Shape(1, 10, 2, 8, 4, 24, 3, 2)
    klr = oracle.build_metadata(sh, K, A)
    base = oracle.predict_select(sh, q, klr, A)["s"]
    for h in range(10):
        q2 = q.copy()
        q2[0, h] = 0.0
        s2 = oracle.predict_select(sh, q2, klr, A)["s"]
        k = h // 5
        assert np.abs(s2[0, k] - base[0, k]).max() > 1e-6
        np.testing.assert_array_equal(s2[0, 1 - k], base[0, 1 - k])


def test_group_to_token_expansion_at_group_size_twelve():
    """Selecting group j must attend tokens 12j .. 12j+11 and nothing else: values planted
    in exactly those rows come back as the output when every key is equal."""
    B, Hq, Hk, d, N, G = 1, 2, 1, 8, 60, 12
    K = np.ones((B, Hk, N, d), np.float32)
    V = np.zeros((B, Hk, N, d), np.float32)
    q = np.ones((B, Hq, d), np.float32)
    j = 3
    V[0, 0, G * j:G * (j + 1)] = 5.0
    V[0, 0, G * j - 1] = -100.0          # neighbours on both sides must stay out
    V[0, 0, G * (j + 1)] = 100.0
    sh = Shape(B, Hq, Hk, d, 4, N, G, 1)
    out = oracle.sparse_attn(sh, q, K, V, np.full((B, Hk, 1), j, np.int32))
    np.testing.assert_allclose(out, 5.0, rtol=0, atol=1e-12)
