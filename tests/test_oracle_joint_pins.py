"""Pins of the oracle's joint-head mode (Sec. 3.2 design (b), the one the paper adopts;
prediction by Eq. 1 with the A_{g(h)} blocks of the single adapter) against things other
than itself.  No GPU needed."""
import numpy as np
import pytest

import oracle
from oracle import Shape
import brute
from workloads import f32_to_bf16_bits, bf16_bits_to_f32


def _problem(seed, B=2, Hq=8, Hk=4, d=8, r=8, N=32, bf16=False):
    g = np.random.default_rng(seed)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    V = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.linalg.qr(g.standard_normal((Hk * d, r)))[0].reshape(Hk, d, r)
    A = np.ascontiguousarray(A.astype(np.float32))
    if bf16:
        K, V, q = (bf16_bits_to_f32(f32_to_bf16_bits(x)) for x in (K, V, q))
    return K, V, q, A


def _store(x, bf16):
    return f32_to_bf16_bits(x) if bf16 else np.ascontiguousarray(x, np.float32)


def _vals(x):
    return (bf16_bits_to_f32(x) if x.dtype == np.uint16 else x).astype(np.float64)


def _shape(B, Hq, Hk, d, r, N, G, M, bf16=False, joint=True, **kw):
    dt = oracle.BF16 if bf16 else oracle.F32
    return Shape(B, Hq, Hk, d, r, N, G, M, kv_dtype=dt, meta_dtype=dt,
                 head_mode=oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE, **kw)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("G", [1, 4, 8])
def test_joint_path_matches_numpy_brute_force(G, bf16):
    B, Hq, Hk, d, r, N = 2, 8, 4, 8, 8, 32
    NG = N // G
    for seed in range(3):
        for M in sorted({1, max(1, NG // 3), NG}):
            K, V, q, A = _problem(seed * 13 + G, B, Hq, Hk, d, r, N, bf16)
            sh = _shape(B, Hq, Hk, d, r, N, G, M, bf16)
            Ks, Vs, qs = _store(K, bf16), _store(V, bf16), _store(q, bf16)
            klr, exact = oracle.build_metadata(sh, Ks, A, want_exact=True)
            assert klr.shape == (B, N, r)
            np.testing.assert_allclose(exact, brute.joint_metadata(K.astype(np.float64), A.astype(np.float64)),
                                       rtol=1e-13, atol=1e-14)
            res = oracle.predict_select(sh, qs, klr, A)
            s_ref = brute.joint_scores(q.astype(np.float64), _vals(klr), A.astype(np.float64))
            np.testing.assert_allclose(res["s"], s_ref, rtol=1e-12, atol=1e-13)
            gs_ref = s_ref.reshape(B, NG, G).max(-1)
            np.testing.assert_allclose(res["gs"], gs_ref, rtol=1e-12, atol=1e-13)
            idx_ref = brute.topk_groups(res["gs"], M)
            assert res["idx"].shape == (B, M)
            np.testing.assert_array_equal(res["idx"], idx_ref)
            # every KV head of the sequence attends the same groups
            rep = np.repeat(idx_ref[:, None, :], Hk, axis=1)
            out = oracle.sparse_attn(sh, qs, Ks, Vs, res["idx"])
            out_ref = brute.sparse_attention(q.astype(np.float64), K.astype(np.float64),
                                             V.astype(np.float64), rep, G)
            np.testing.assert_allclose(out, out_ref, rtol=1e-12, atol=1e-13)


def test_one_kv_head_makes_both_modes_coincide():
    # with H_kv = 1 the flattened row IS the head's row and "all heads" ARE the heads of
    # that KV head: the two designs of Sec. 3.2 are the same computation
    B, Hq, Hk, d, r, N, G, M = 2, 4, 1, 8, 4, 64, 4, 5
    K, V, q, A = _problem(3, B, Hq, Hk, d, r, N)
    j = _shape(B, Hq, Hk, d, r, N, G, M, joint=True)
    s = _shape(B, Hq, Hk, d, r, N, G, M, joint=False)
    kj = oracle.build_metadata(j, K, A)
    ks = oracle.build_metadata(s, K, A)
    np.testing.assert_array_equal(kj, ks[:, 0])
    rj, rs = oracle.predict_select(j, q, kj, A), oracle.predict_select(s, q, ks, A)
    np.testing.assert_array_equal(rj["s"], rs["s"][:, 0])
    np.testing.assert_array_equal(rj["idx"], rs["idx"][:, 0])
    np.testing.assert_array_equal(oracle.sparse_attn(j, q, K, V, rj["idx"]),
                                  oracle.sparse_attn(s, q, K, V, rs["idx"]))


def test_block_diagonal_adapter_gives_the_sum_of_the_per_head_scores():
    # A = blockdiag(A_0 .. A_{H-1}): Flatten(K).A is the concatenation of the per-head K_lr
    # and (q_h A_{g(h)}) only meets the columns of its own head, so the joint token score is
    # the sum over KV heads of the per-head design's scores
    B, Hq, Hk, d, rh, N, G, M = 2, 8, 4, 8, 2, 32, 4, 3
    g = np.random.default_rng(5)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    Ah = g.standard_normal((Hk, d, rh)).astype(np.float32)
    Aj = np.zeros((Hk, d, Hk * rh), np.float32)
    for k in range(Hk):
        Aj[k, :, k * rh:(k + 1) * rh] = Ah[k]
    sep = _shape(B, Hq, Hk, d, rh, N, G, M, joint=False)
    jnt = _shape(B, Hq, Hk, d, Hk * rh, N, G, M, joint=True)
    k_sep, e_sep = oracle.build_metadata(sep, K, Ah, want_exact=True)
    k_jnt, e_jnt = oracle.build_metadata(jnt, K, Aj, want_exact=True)
    np.testing.assert_array_equal(e_jnt, np.concatenate([e_sep[:, k] for k in range(Hk)], axis=-1))
    s_sep = oracle.predict_select(sep, q, k_sep, Ah)["s"]
    s_jnt = oracle.predict_select(jnt, q, k_jnt, Aj)["s"]
    np.testing.assert_allclose(s_jnt, s_sep.sum(axis=1), rtol=1e-12, atol=1e-12)


def test_identity_adapter_gives_the_sum_of_exact_logits_of_all_heads():
    # r = H_kv d and A = I: K_lr is the flattened cache itself and Eq. (1) is exact, so the
    # token score is sum_h q_h . K_{g(h)}[n]
    B, Hq, Hk, d, N, G, M = 2, 4, 2, 8, 32, 4, 2
    g = np.random.default_rng(7)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.eye(Hk * d, dtype=np.float32).reshape(Hk, d, Hk * d)
    sh = _shape(B, Hq, Hk, d, Hk * d, N, G, M)
    klr = oracle.build_metadata(sh, K, A)
    np.testing.assert_array_equal(klr, brute.flatten_keys(K))
    s = oracle.predict_select(sh, q, klr, A)["s"]
    qpk = Hq // Hk
    exact = np.zeros((B, N))
    for h in range(Hq):
        exact += np.einsum("bd,bnd->bn", q[:, h].astype(np.float64), K[:, h // qpk].astype(np.float64))
    np.testing.assert_allclose(s, exact, rtol=1e-12, atol=1e-12)


def test_each_head_uses_the_block_of_its_own_kv_head():
    # zeroing the queries of the heads of KV head 1 must leave exactly the contribution of
    # the A_0 block; swapping the blocks must change it (guards g(h) and the row ranges)
    B, Hq, Hk, d, r, N, G, M = 1, 4, 2, 8, 4, 16, 2, 1
    K, V, q, A = _problem(11, B, Hq, Hk, d, r, N)
    sh = _shape(B, Hq, Hk, d, r, N, G, M)
    klr = oracle.build_metadata(sh, K, A)
    q0 = q.copy()
    q0[:, 2:] = 0
    s = oracle.predict_select(sh, q0, klr, A)["s"]
    want = np.einsum("bhd,dr,bnr->bn", q0[:, :2].astype(np.float64), A[0].astype(np.float64),
                     klr.astype(np.float64))
    np.testing.assert_allclose(s, want, rtol=1e-12, atol=1e-13)
    s_swapped = oracle.predict_select(sh, q0, klr, np.ascontiguousarray(A[::-1]))["s"]
    assert np.abs(s_swapped - s).max() > 1e-3


def test_shared_selection_equals_replicated_selection():
    B, Hq, Hk, d, r, N, G, M = 2, 8, 4, 8, 8, 64, 4, 6
    K, V, q, A = _problem(13, B, Hq, Hk, d, r, N)
    g = np.random.default_rng(1)
    idx = np.stack([np.sort(g.choice(N // G, M, replace=False)) for _ in range(B)]).astype(np.int32)
    j = oracle.sparse_attn(_shape(B, Hq, Hk, d, r, N, G, M, joint=True), q, K, V, idx)
    s = oracle.sparse_attn(_shape(B, Hq, Hk, d, r, N, G, M, joint=False), q, K, V,
                           np.ascontiguousarray(np.repeat(idx[:, None], Hk, axis=1)))
    np.testing.assert_array_equal(j, s)


def test_joint_selecting_every_group_equals_dense_attention_and_threads_agree():
    B, Hq, Hk, d, r, N, G = 2, 8, 4, 8, 8, 32, 4
    K, V, q, A = _problem(17, B, Hq, Hk, d, r, N)
    sh = _shape(B, Hq, Hk, d, r, N, G, N // G)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    np.testing.assert_array_equal(res["idx"], np.tile(np.arange(N // G, dtype=np.int32), (B, 1)))
    np.testing.assert_allclose(oracle.sparse_attn(sh, q, K, V, res["idx"]), oracle.dense_attn(sh, q, K, V),
                               rtol=1e-13, atol=1e-14)
    sh4 = _shape(B, Hq, Hk, d, r, N, G, 3, n_threads=4)
    sh1 = _shape(B, Hq, Hk, d, r, N, G, 3)
    a, b = oracle.predict_select(sh4, q, klr, A), oracle.predict_select(sh1, q, klr, A)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["s"], b["s"])


def test_unknown_head_mode_is_rejected():
    K, V, q, A = _problem(1)
    sh = Shape(2, 8, 4, 8, 8, 32, 4, 2, head_mode=7)
    with pytest.raises(RuntimeError):
        oracle.build_metadata(Shape(**{**sh.__dict__}), K, A)
