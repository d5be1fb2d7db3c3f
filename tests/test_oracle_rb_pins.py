"""Pins of the oracle's rolling buffer (Sec. 3.4.1: the newest tokens, not yet a complete
group, are kept outside the cache, never scored, always attended), of the row capacity of
the cache arrays, and of the metadata of a row range -- against things other than itself."""
import numpy as np
import pytest

import oracle
from oracle import Shape
import brute
from workloads import f32_to_bf16_bits, bf16_bits_to_f32


def _problem(seed, B=2, Hq=4, Hk=2, d=8, r=4, N=32, cap_rb=6):
    g = np.random.default_rng(seed)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    V = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.ascontiguousarray(g.standard_normal((Hk, d, r)).astype(np.float32))
    rbK = g.standard_normal((B, Hk, cap_rb, d)).astype(np.float32)
    rbV = g.standard_normal((B, Hk, cap_rb, d)).astype(np.float32)
    return K, V, q, A, rbK, rbV


def _rand_idx(seed, lead, NG, M):
    g = np.random.default_rng(seed)
    n = int(np.prod(lead))
    return np.stack([np.sort(g.choice(NG, M, replace=False)) for _ in range(n)]).astype(np.int32).reshape(lead + (M,))


@pytest.mark.parametrize("joint", [False, True])
@pytest.mark.parametrize("rb_len", [1, 3, 6])
def test_buffer_tokens_join_one_softmax_with_the_selected_tokens(rb_len, joint):
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 32, 4, 3
    K, V, q, A, rbK, rbV = _problem(rb_len)
    sh = Shape(B, Hq, Hk, d, 4, N, G, M, head_mode=oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE)
    idx = _rand_idx(5, sh.sets, N // G, M)
    out = oracle.sparse_attn(sh, q, K, V, idx, rbK, rbV, rb_len)
    # brute force: dense attention over the concatenation [selected rows ; buffer rows]
    per_head = idx if not joint else np.repeat(idx[:, None], Hk, axis=1)
    Kc = np.concatenate([K, rbK[:, :, :rb_len]], axis=2).astype(np.float64)
    Vc = np.concatenate([V, rbV[:, :, :rb_len]], axis=2).astype(np.float64)
    toks = [[np.concatenate([(per_head[b, k][:, None] * G + np.arange(G)).ravel(), N + np.arange(rb_len)])
             for k in range(Hk)] for b in range(B)]
    ref = brute.attention_over_tokens(q.astype(np.float64), Kc, Vc, toks)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    # rows of the buffer past rb_len are never read
    rbK2, rbV2 = rbK.copy(), rbV.copy()
    rbK2[:, :, rb_len:] = np.nan
    rbV2[:, :, rb_len:] = np.nan
    np.testing.assert_array_equal(oracle.sparse_attn(sh, q, K, V, idx, rbK2, rbV2, rb_len), out)


def test_empty_buffer_changes_nothing():
    K, V, q, A, rbK, rbV = _problem(2)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    idx = _rand_idx(1, sh.sets, 8, 3)
    np.testing.assert_array_equal(oracle.sparse_attn(sh, q, K, V, idx, rbK, rbV, 0),
                                  oracle.sparse_attn(sh, q, K, V, idx))


def test_a_cache_group_moved_into_the_buffer_gives_the_same_output():
    # attention is a function of the SET of attended tokens: the last group attended from
    # the cache, or the same rows attended from the buffer, must agree
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 32, 4, 3
    K, V, q, A, _, _ = _problem(3)
    NG = N // G
    base = _rand_idx(2, (B, Hk), NG - 1, M - 1)               # groups other than the last
    with_last = np.concatenate([base, np.full((B, Hk, 1), NG - 1, np.int32)], axis=-1)
    a = oracle.sparse_attn(Shape(B, Hq, Hk, d, 4, N, G, M), q, K, V, with_last)
    rbK = np.ascontiguousarray(K[:, :, N - G:])
    rbV = np.ascontiguousarray(V[:, :, N - G:])
    b = oracle.sparse_attn(Shape(B, Hq, Hk, d, 4, N, G, M - 1), q, K, V, base, rbK, rbV, G)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)


def test_all_groups_plus_buffer_is_dense_attention_over_the_longer_cache():
    B, Hq, Hk, d, N, G = 2, 4, 2, 8, 32, 4
    K, V, q, A, rbK, rbV = _problem(4)
    T = 3
    idx = np.tile(np.arange(N // G, dtype=np.int32), (B, Hk, 1))
    a = oracle.sparse_attn(Shape(B, Hq, Hk, d, 4, N, G, N // G), q, K, V, idx, rbK, rbV, T)
    Kc = np.ascontiguousarray(np.concatenate([K, rbK[:, :, :T]], axis=2))
    Vc = np.ascontiguousarray(np.concatenate([V, rbV[:, :, :T]], axis=2))
    dense = brute.dense_attention(q.astype(np.float64), Kc.astype(np.float64), Vc.astype(np.float64))
    np.testing.assert_allclose(a, dense, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("joint", [False, True])
def test_padded_arrays_with_poisoned_padding_give_the_compact_results(joint):
    B, Hq, Hk, d, r, N, G, M, cap = 2, 4, 2, 8, 4, 32, 4, 3, 44
    K, V, q, A, rbK, rbV = _problem(6)
    mode = oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE
    sh = Shape(B, Hq, Hk, d, r, N, G, M, head_mode=mode)
    shp = Shape(B, Hq, Hk, d, r, N, G, M, head_mode=mode, ctx_capacity=cap)

    def pad(x, fill):
        out = np.full(x.shape[:-2] + (cap, x.shape[-1]), fill, dtype=x.dtype)
        out[..., :N, :] = x
        return out

    klr = oracle.build_metadata(sh, K, A)
    klr_p = oracle.build_metadata(shp, pad(K, np.nan), A)
    np.testing.assert_array_equal(klr_p[..., :N, :], klr)
    assert not np.any(klr_p[..., N:, :])                      # rows past ctx_len are not written
    ref = oracle.predict_select(sh, q, klr, A)
    got = oracle.predict_select(shp, q, pad(klr, np.nan), A)
    for key in ("idx", "gs", "s", "boundary"):
        np.testing.assert_array_equal(got[key], ref[key])
    np.testing.assert_array_equal(
        oracle.sparse_attn(shp, q, pad(K, np.nan), pad(V, np.nan), ref["idx"], rbK, rbV, 2),
        oracle.sparse_attn(sh, q, K, V, ref["idx"], rbK, rbV, 2))
    np.testing.assert_array_equal(oracle.dense_attn(shp, q, pad(K, np.nan), pad(V, np.nan)),
                                  oracle.dense_attn(sh, q, K, V))


@pytest.mark.parametrize("joint", [False, True])
def test_metadata_of_a_row_range_equals_those_rows_of_the_full_build(joint):
    # appending a completed group: rows [N, N+G) of a cache with spare capacity
    B, Hq, Hk, d, r, N, G, cap = 2, 4, 2, 8, 4, 24, 4, 32
    g = np.random.default_rng(8)
    K = g.standard_normal((B, Hk, cap, d)).astype(np.float32)
    A = np.ascontiguousarray(g.standard_normal((Hk, d, r)).astype(np.float32))
    mode = oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE
    full = oracle.build_metadata(Shape(B, Hq, Hk, d, r, cap, G, 1, head_mode=mode), K, A)
    sh = Shape(B, Hq, Hk, d, r, N, G, 1, head_mode=mode, ctx_capacity=cap)
    klr = oracle.build_metadata(sh, K, A)
    np.testing.assert_array_equal(klr[..., :N, :], full[..., :N, :])
    oracle.build_metadata_rows(sh, K, A, klr, N, G)
    np.testing.assert_array_equal(klr[..., :N + G, :], full[..., :N + G, :])
    assert not np.any(klr[..., N + G:, :])
    with pytest.raises(RuntimeError):
        oracle.build_metadata_rows(sh, K, A, klr, cap - 2, G)     # leaves the capacity


def test_bad_buffer_arguments_are_rejected():
    K, V, q, A, rbK, rbV = _problem(9)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    idx = _rand_idx(1, sh.sets, 8, 3)
    with pytest.raises(RuntimeError):
        oracle.sparse_attn(sh, q, K, V, idx, rbK, rbV, 7)          # rb_len > capacity
    with pytest.raises(RuntimeError):
        oracle.build_metadata(Shape(2, 4, 2, 8, 4, 32, 4, 3, ctx_capacity=16),
                              np.ascontiguousarray(K[:, :, :16]), A)                 # capacity < ctx_len
