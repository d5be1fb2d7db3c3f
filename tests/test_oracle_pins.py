"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the statement of the paper (or the piece of mathematics) that
fixes the expected value.  A plausible slip in the oracle -- a dropped head in
the sum, A used transposed, max taken over the wrong axis, a wrong tie rule,
a missing softmax scale, an off-by-one in the group -> token expansion --
breaks at least one of them.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import Shape
import brute
from workloads import f32_to_bf16_bits, bf16_bits_to_f32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(seed, B=2, Hq=4, Hk=2, d=8, r=4, N=32, bf16=False, orth=True):
    g = np.random.default_rng(seed)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    V = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = g.standard_normal((Hk, d, r))
    if orth:
        A = np.stack([np.linalg.qr(A[k])[0] for k in range(Hk)])
    A = np.ascontiguousarray(A.astype(np.float32))
    if bf16:
        K, V, q = (bf16_bits_to_f32(f32_to_bf16_bits(x)) for x in (K, V, q))
    return K, V, q, A


def _store(x, bf16):
    return f32_to_bf16_bits(x) if bf16 else np.ascontiguousarray(x, np.float32)


def _vals(x):
    return (bf16_bits_to_f32(x) if x.dtype == np.uint16 else x).astype(np.float64)


# --------------------------------------------------------------------------
# whole path vs the independent numpy brute force (tiny shapes, many cases)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_whole_path_matches_numpy_brute_force(G, bf16):
    N, d, r = 32, 8, 4
    NG = N // G
    for seed, M in itertools.product(range(4), sorted({1, 3 if NG > 3 else 1, NG - 1, NG})):
        if M < 1:
            continue
        K, V, q, A = _rand_problem(seed * 17 + G, d=d, r=r, N=N, bf16=bf16)
        dt = oracle.BF16 if bf16 else oracle.F32
        sh = Shape(2, 4, 2, d, r, N, G, M, kv_dtype=dt, meta_dtype=dt)
        Ks, Vs, qs = _store(K, bf16), _store(V, bf16), _store(q, bf16)

        klr, exact = oracle.build_metadata(sh, Ks, A, want_exact=True)
        ref_exact = np.einsum("bknd,kdr->bknr", K.astype(np.float64), A.astype(np.float64))
        np.testing.assert_allclose(exact, ref_exact, rtol=1e-13, atol=1e-14)

        res = oracle.predict_select(sh, qs, klr, A)
        s_ref = brute.scores(q.astype(np.float64), _vals(klr), A.astype(np.float64))
        np.testing.assert_allclose(res["s"], s_ref, rtol=1e-12, atol=1e-13)
        gs_ref = brute.group_scores(s_ref, G)
        np.testing.assert_allclose(res["gs"], gs_ref, rtol=1e-12, atol=1e-13)
        # index parity is judged on the oracle's own scores (identical up to 1e-13,
        # far below any gap between random scores)
        idx_ref = brute.topk_groups(res["gs"], M)
        np.testing.assert_array_equal(res["idx"], idx_ref)

        out = oracle.sparse_attn(sh, qs, Ks, Vs, res["idx"])
        out_ref = brute.sparse_attention(q.astype(np.float64), K.astype(np.float64),
                                         V.astype(np.float64), idx_ref, G)
        np.testing.assert_allclose(out, out_ref, rtol=1e-12, atol=1e-13)


def test_mean_reduce_matches_brute_force():
    K, V, q, A = _rand_problem(5)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3, reduce=oracle.REDUCE_MEAN)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    s_ref = brute.scores(q.astype(np.float64), klr.astype(np.float64), A.astype(np.float64))
    gs_ref = brute.group_scores(s_ref, 4, mean=True)
    np.testing.assert_allclose(res["gs"], gs_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(res["idx"], brute.topk_groups(res["gs"], 3))
    # mean and max must differ on random data (guards against the flag being ignored)
    res_max = oracle.predict_select(Shape(2, 4, 2, 8, 4, 32, 4, 3), q, klr, A)
    assert np.abs(res_max["gs"] - res["gs"]).max() > 1e-3


# --------------------------------------------------------------------------
# metadata construction, Sec. 3.2: K_lr = K . A
# --------------------------------------------------------------------------
def test_build_metadata_with_selection_adapter_copies_columns():
    """A whose column j is the unit vector e_perm[j] makes K_lr[n, j] = K[n, perm[j]]
    exactly.  d != r, so using A transposed, or indexing it [j, i], cannot pass."""
    g = np.random.default_rng(0)
    B, Hk, N, d, r = 2, 3, 12, 8, 4
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    A = np.zeros((Hk, d, r), np.float32)
    perms = [g.permutation(d)[:r] for _ in range(Hk)]
    for k in range(Hk):
        A[k, perms[k], np.arange(r)] = 1.0
    sh = Shape(B, 2 * Hk, Hk, d, r, N, 4, 1)
    klr = oracle.build_metadata(sh, K, A)
    for k in range(Hk):
        np.testing.assert_array_equal(klr[:, k], K[:, k][:, :, perms[k]])


def _nearest_bf16_by_search(x: float) -> int:
    """Nearest bf16 to a double by comparing the neighbouring bit patterns."""
    base = int(f32_to_bf16_bits(np.array([x], np.float32))[0])
    best = None
    for cand in range(max(base - 2, 0), base + 3):
        v = float(bf16_bits_to_f32(np.array([cand], np.uint16))[0])
        if not np.isfinite(v) or (v != 0 and np.sign(v) != np.sign(x)):
            continue
        err = abs(v - x)
        key = (err, cand & 1)  # smaller error first, then even mantissa
        if best is None or key < best[0]:
            best = (key, cand)
    return best[1]


def test_bf16_rounding_hand_derived_values():
    """bf16 keeps 8 significant bits: the spacing in [1, 2) is 2^-7.
    1 + 2^-8 is halfway between 1 (mantissa 0, even) and 1 + 2^-7 (odd) -> 1.
    1 + 3*2^-8 is halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even) -> 1 + 2^-6."""
    assert oracle.round_to_bf16(1.0) == 0x3F80
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81  # just above the midpoint
    assert oracle.round_to_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 0xBF81
    assert oracle.round_to_bf16(0.0) == 0x0000
    assert oracle.round_to_bf16(2.0 - 2.0 ** -9) == 0x4000  # rounds up into the next binade
    assert oracle.round_to_bf16(3.140625) == 0x4049
    assert oracle.round_to_bf16(0.1) == 0x3DCD  # 0.1 = 0x3DCCCCCD in fp32


def test_bf16_rounding_matches_neighbour_search_and_torch():
    g = np.random.default_rng(1)
    xs = np.concatenate([g.standard_normal(300) * 10.0 ** g.integers(-6, 6, 300),
                         [2.0 ** -130, 1e-38, 65504.0, 3.3e38]])
    for x in xs:
        assert oracle.round_to_bf16(float(x)) == _nearest_bf16_by_search(float(x)), x
    torch = pytest.importorskip("torch")
    x32 = (g.standard_normal(4096) * 3).astype(np.float32)
    ref = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.round_to_bf16(float(v)) for v in x32], dtype=np.uint16)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(f32_to_bf16_bits(x32), ref)  # the generator's cast as well


# --------------------------------------------------------------------------
# prediction, Sec. 3.3 / Eq. (1)
# --------------------------------------------------------------------------
def test_identity_adapter_gives_exact_qk_scores():
    """r = d and A = I: K_lr = K and the token importance is sum_h q_h . K[n] exactly."""
    B, Hq, Hk, d, N = 2, 6, 2, 8, 24
    K, V, q, _ = _rand_problem(3, B=B, Hq=Hq, Hk=Hk, d=d, r=d, N=N)
    A = np.stack([np.eye(d, dtype=np.float32)] * Hk)
    sh = Shape(B, Hq, Hk, d, d, N, 4, 2)
    klr = oracle.build_metadata(sh, K, A)
    np.testing.assert_array_equal(klr, K)
    res = oracle.predict_select(sh, q, klr, A)
    qsum = q.astype(np.float64).reshape(B, Hk, Hq // Hk, d)
    exact = np.einsum("bkhd,bknd->bkn", qsum, K.astype(np.float64))
    np.testing.assert_allclose(res["s"], exact, rtol=1e-12, atol=1e-13)


def test_orthogonal_full_rank_adapter_gives_exact_scores():
    """Any orthogonal A with r = d has A A^T = I, so (q A)(K A)^T = q K^T (Eq. 1 is exact)."""
    B, Hq, Hk, d, N = 1, 4, 2, 8, 16
    K, V, q, A = _rand_problem(4, B=B, Hq=Hq, Hk=Hk, d=d, r=d, N=N, orth=True)
    sh = Shape(B, Hq, Hk, d, d, N, 2, 2)
    _, exact_klr = oracle.build_metadata(sh, K, A, want_exact=True)
    # feed the metadata in fp32 storage: rounding of K_lr bounds the error at ~1e-6
    res = oracle.predict_select(sh, q, exact_klr.astype(np.float32), A)
    qsum = q.astype(np.float64).reshape(B, Hk, Hq // Hk, d)
    exact = np.einsum("bkhd,bknd->bkn", qsum, K.astype(np.float64))
    np.testing.assert_allclose(res["s"], exact, rtol=0, atol=2e-5)


def test_exactly_low_rank_keys_give_exact_scores():
    """Keys that lie in the span of A's columns (here: only the coordinates A selects
    are non-zero) are reproduced exactly by the rank-r metadata."""
    g = np.random.default_rng(6)
    B, Hq, Hk, d, r, N = 1, 4, 2, 8, 3, 16
    sel = [np.array([1, 4, 6]), np.array([0, 2, 7])]
    K = np.zeros((B, Hk, N, d), np.float32)
    A = np.zeros((Hk, d, r), np.float32)
    for k in range(Hk):
        K[:, k][:, :, sel[k]] = g.standard_normal((B, N, r)).astype(np.float32)
        A[k, sel[k], np.arange(r)] = 1.0
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    sh = Shape(B, Hq, Hk, d, r, N, 4, 1)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    qsum = q.astype(np.float64).reshape(B, Hk, Hq // Hk, d)
    exact = np.einsum("bkhd,bknd->bkn", qsum, K.astype(np.float64))
    np.testing.assert_allclose(res["s"], exact, rtol=1e-12, atol=1e-13)


def test_both_sides_of_eq1_agree():
    """(Q_h A) K_lr^T  ==  Q_h (K_lr A^T)^T, the identity printed as Eq. (1)."""
    K, V, q, A = _rand_problem(7, orth=False)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 2)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    A64, klr64, q64 = A.astype(np.float64), klr.astype(np.float64), q.astype(np.float64)
    recon = np.einsum("bknr,kdr->bknd", klr64, A64)          # K_lr A^T: reconstructed keys
    rhs = np.einsum("bkhd,bknd->bkn", q64.reshape(2, 2, 2, 8), recon)
    np.testing.assert_allclose(res["s"], rhs, rtol=1e-11, atol=1e-12)


def test_head_sum_covers_exactly_the_heads_of_the_kv_head():
    """Zeroing the queries of the heads mapped to KV head 0 must zero KV head 0's scores
    and leave KV head 1's untouched (g(h) = h // (H_q/H_kv))."""
    K, V, q, A = _rand_problem(8, Hq=6, Hk=2)
    sh = Shape(2, 6, 2, 8, 4, 32, 4, 2)
    klr = oracle.build_metadata(sh, K, A)
    base = oracle.predict_select(sh, q, klr, A)["s"]
    q0 = q.copy()
    q0[:, 0:3] = 0
    s0 = oracle.predict_select(sh, q0, klr, A)["s"]
    assert np.all(s0[:, 0] == 0)
    np.testing.assert_array_equal(s0[:, 1], base[:, 1])
    # and every head of a KV head contributes: dropping one head changes the score
    q1 = q.copy()
    q1[:, 2] = 0
    assert np.abs(oracle.predict_select(sh, q1, klr, A)["s"][:, 0] - base[:, 0]).max() > 1e-3


def test_group_size_one_is_plain_token_topk():
    K, V, q, A = _rand_problem(9)
    sh = Shape(2, 4, 2, 8, 4, 32, 1, 5)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    np.testing.assert_array_equal(res["gs"], res["s"])
    np.testing.assert_array_equal(res["idx"], brute.topk_groups(res["s"], 5))


def test_group_max_dominates_members_and_spike_ranks_first():
    K, V, q, A = _rand_problem(10, B=1, Hq=2, Hk=1)
    sh = Shape(1, 2, 1, 8, 4, 32, 4, 1)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    s, gs = res["s"][0, 0], res["gs"][0, 0]
    assert np.all(gs[:, None] >= s.reshape(8, 4))
    assert np.all(gs == s.reshape(8, 4).max(1))
    # plant a spike: make token 22 (group 5) a copy of the low-rank query direction
    q_lr = np.einsum("hd,dr->r", q[0].astype(np.float64), A[0].astype(np.float64))
    klr2 = klr.copy()
    klr2[0, 0, 22] = (100.0 * q_lr / np.linalg.norm(q_lr)).astype(np.float32)
    res2 = oracle.predict_select(sh, q, klr2, A)
    assert res2["idx"][0, 0, 0] == 5
    assert res2["boundary"][0, 0, 0] == res2["gs"][0, 0, 5]


def test_selection_is_invariant_to_power_of_two_query_scaling():
    K, V, q, A = _rand_problem(11)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    klr = oracle.build_metadata(sh, K, A)
    a = oracle.predict_select(sh, q, klr, A)
    b = oracle.predict_select(sh, q * np.float32(8.0), klr, A)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["gs"] * 8.0, b["gs"])


def test_ties_resolve_to_the_lower_index_and_output_is_ascending():
    B, Hq, Hk, d, r, N, G = 1, 2, 1, 4, 2, 40, 4
    g = np.random.default_rng(12)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.ascontiguousarray(np.linalg.qr(g.standard_normal((d, r)))[0][None].astype(np.float32))
    # all rows identical -> all 10 group scores exactly equal -> first M groups win
    klr = np.tile(g.standard_normal((1, 1, 1, r)).astype(np.float32), (1, 1, N, 1))
    for M in (1, 3, 10):
        res = oracle.predict_select(Shape(B, Hq, Hk, d, r, N, G, M), q, klr, A)
        np.testing.assert_array_equal(res["idx"][0, 0], np.arange(M))
    # two identical groups at the selection boundary: only the earlier one is taken
    klr = g.standard_normal((1, 1, N, r)).astype(np.float32)
    klr[0, 0, 7 * G:8 * G] = klr[0, 0, 2 * G:3 * G]
    res_all = oracle.predict_select(Shape(B, Hq, Hk, d, r, N, G, 10), q, klr, A)
    gs = res_all["gs"][0, 0]
    assert gs[2] == gs[7]
    M = int((gs > gs[2]).sum()) + 1
    res = oracle.predict_select(Shape(B, Hq, Hk, d, r, N, G, M), q, klr, A)
    sel = res["idx"][0, 0]
    assert 2 in sel and 7 not in sel
    assert np.all(np.diff(sel) > 0)
    assert res["boundary"][0, 0, 0] == res["boundary"][0, 0, 1] == gs[2]


def test_boundary_reports_mth_and_next_score():
    K, V, q, A = _rand_problem(13)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    klr = oracle.build_metadata(sh, K, A)
    res = oracle.predict_select(sh, q, klr, A)
    srt = -np.sort(-res["gs"], axis=-1)
    np.testing.assert_array_equal(res["boundary"][..., 0], srt[..., 2])
    np.testing.assert_array_equal(res["boundary"][..., 1], srt[..., 3])
    full = oracle.predict_select(Shape(2, 4, 2, 8, 4, 32, 4, 8), q, klr, A)
    np.testing.assert_array_equal(full["idx"], np.tile(np.arange(8, dtype=np.int32), (2, 2, 1)))
    assert np.all(np.isneginf(full["boundary"][..., 1]))


# --------------------------------------------------------------------------
# attention over the selected groups
# --------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
def test_selecting_every_group_equals_dense_attention(bf16):
    K, V, q, A = _rand_problem(14, bf16=bf16)
    dt = oracle.BF16 if bf16 else oracle.F32
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 8, kv_dtype=dt, meta_dtype=dt)
    Ks, Vs, qs = _store(K, bf16), _store(V, bf16), _store(q, bf16)
    idx = np.tile(np.arange(8, dtype=np.int32), (2, 2, 1))
    sparse = oracle.sparse_attn(sh, qs, Ks, Vs, idx)
    dense = oracle.dense_attn(sh, qs, Ks, Vs)
    np.testing.assert_allclose(sparse, dense, rtol=1e-13, atol=1e-14)
    ref = brute.dense_attention(q.astype(np.float64), K.astype(np.float64), V.astype(np.float64))
    np.testing.assert_allclose(dense, ref, rtol=1e-12, atol=1e-13)
    # library routine: torch's scaled_dot_product_attention in fp64
    torch = pytest.importorskip("torch")
    tq = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    tk = torch.from_numpy(K.astype(np.float64)).repeat_interleave(2, dim=1)
    tv = torch.from_numpy(V.astype(np.float64)).repeat_interleave(2, dim=1)
    sdpa = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0, :].numpy()
    np.testing.assert_allclose(dense, sdpa, rtol=1e-10, atol=1e-12)


def test_sparse_attention_is_order_independent_and_uses_only_selected_tokens():
    K, V, q, A = _rand_problem(15)
    sh = Shape(2, 4, 2, 8, 4, 32, 4, 3)
    idx = np.array([[[1, 4, 6], [0, 2, 7]], [[3, 5, 6], [1, 2, 3]]], np.int32)
    out = oracle.sparse_attn(sh, q, K, V, idx)
    out_perm = oracle.sparse_attn(sh, q, K, V, np.ascontiguousarray(idx[..., ::-1]))
    np.testing.assert_allclose(out, out_perm, rtol=1e-13, atol=1e-15)
    # poison every unselected token: the result must not move
    K2, V2 = K.copy(), V.copy()
    for b in range(2):
        for k in range(2):
            mask = np.ones(32, bool)
            for j in idx[b, k]:
                mask[j * 4:(j + 1) * 4] = False
            K2[b, k, mask] = 1e6
            V2[b, k, mask] = -1e6
    np.testing.assert_array_equal(oracle.sparse_attn(sh, q, K2, V2, idx), out)
    # each output component is a convex combination of the selected V rows
    for b in range(2):
        for h in range(4):
            k = h // 2
            rows = np.concatenate([np.arange(j * 4, j * 4 + 4) for j in idx[b, k]])
            assert np.all(out[b, h] <= V[b, k, rows].max(0) + 1e-12)
            assert np.all(out[b, h] >= V[b, k, rows].min(0) - 1e-12)


def test_closed_form_attention_cases():
    """Hand-derived cases of softmax attention (Sec. 2.1), one per line of
    tests/golden/closed_form_attention.txt: d = 1, q = 1, scale = 1, keys k0, k1
    and values v0, v1; the output is (e^k0 v0 + e^k1 v1) / (e^k0 + e^k1)."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "closed_form_attention.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 4
    for k0, k1, v0, v1, expect, tol in rows:
        K = np.array([float(k0), float(k1)], np.float32).reshape(1, 1, 2, 1)
        V = np.array([float(v0), float(v1)], np.float32).reshape(1, 1, 2, 1)
        q = np.ones((1, 1, 1), np.float32)
        sh = Shape(1, 1, 1, 1, 1, 2, 2, 1, softmax_scale=1.0)
        out = oracle.sparse_attn(sh, q, K, V, np.zeros((1, 1, 1), np.int32))
        assert abs(out[0, 0, 0] - float(expect)) <= float(tol), (k0, k1, v0, v1)


def test_default_scale_is_inverse_sqrt_d_and_identical_keys_average_values():
    g = np.random.default_rng(16)
    d, N = 16, 8
    # identical keys: uniform weights whatever the scale -> mean of the selected V rows
    K = np.tile(g.standard_normal((1, 1, 1, d)).astype(np.float32), (1, 1, N, 1))
    V = g.standard_normal((1, 1, N, d)).astype(np.float32)
    q = g.standard_normal((1, 1, d)).astype(np.float32)
    sh = Shape(1, 1, 1, d, 4, N, 2, 2)
    out = oracle.sparse_attn(sh, q, K, V, np.array([[[1, 3]]], np.int32))
    np.testing.assert_allclose(out[0, 0], V[0, 0, [2, 3, 6, 7]].astype(np.float64).mean(0),
                               rtol=1e-13, atol=1e-15)
    # scale: with d = 16 the default is 1/4, so multiplying q by 4 and passing scale = 1/16
    # is the same computation (all quantities exact in fp32)
    K = g.standard_normal((1, 1, N, d)).astype(np.float32)
    a = oracle.dense_attn(Shape(1, 1, 1, d, 4, N, 2, 2), q, K, V)
    b = oracle.dense_attn(Shape(1, 1, 1, d, 4, N, 2, 2, softmax_scale=0.25), q, K, V)
    c = oracle.dense_attn(Shape(1, 1, 1, d, 4, N, 2, 2, softmax_scale=1.0 / 16), q * np.float32(4), K, V)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_allclose(a, c, rtol=1e-13, atol=1e-15)
    unscaled = oracle.dense_attn(Shape(1, 1, 1, d, 4, N, 2, 2, softmax_scale=1.0), q, K, V)
    assert np.abs(unscaled - a).max() > 1e-3


def test_softmax_shift_invariance():
    """Adding the same vector u to every key shifts all logits by q.u and leaves the
    attention output unchanged.  Small integers keep every stored value exact."""
    g = np.random.default_rng(17)
    d, N = 8, 16
    K = g.integers(-3, 4, (1, 1, N, d)).astype(np.float32)
    V = g.standard_normal((1, 1, N, d)).astype(np.float32)
    q = g.integers(-2, 3, (1, 2, d)).astype(np.float32)
    u = g.integers(-5, 6, d).astype(np.float32)
    sh = Shape(1, 2, 1, d, 2, N, 4, 2)
    idx = np.array([[[0, 3]]], np.int32)
    a = oracle.sparse_attn(sh, q, K, V, idx)
    b = oracle.sparse_attn(sh, q, K + u, V, idx)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_threaded_run_is_identical_to_serial():
    K, V, q, A = _rand_problem(18, B=3, Hq=8, Hk=4, N=64)
    sh1 = Shape(3, 8, 4, 8, 4, 64, 4, 5)
    sh4 = Shape(3, 8, 4, 8, 4, 64, 4, 5, n_threads=4)
    k1, k4 = oracle.build_metadata(sh1, K, A), oracle.build_metadata(sh4, K, A)
    np.testing.assert_array_equal(k1, k4)
    r1, r4 = oracle.predict_select(sh1, q, k1, A), oracle.predict_select(sh4, q, k1, A)
    for key in r1:
        np.testing.assert_array_equal(r1[key], r4[key])
    np.testing.assert_array_equal(oracle.sparse_attn(sh1, q, K, V, r1["idx"]),
                                  oracle.sparse_attn(sh4, q, K, V, r1["idx"]))


def test_bad_parameters_are_rejected():
    K, V, q, A = _rand_problem(19)
    klr = oracle.build_metadata(Shape(2, 4, 2, 8, 4, 32, 4, 3), K, A)
    with pytest.raises(RuntimeError):   # M > NG
        oracle.predict_select(Shape(2, 4, 2, 8, 4, 32, 4, 9), q, klr, A)
    with pytest.raises(RuntimeError):   # group index out of range
        oracle.sparse_attn(Shape(2, 4, 2, 8, 4, 32, 4, 1), q, K, V, np.full((2, 2, 1), 8, np.int32))
    bad = Shape(2, 4, 2, 8, 4, 30, 4, 3)  # N % G != 0
    with pytest.raises(RuntimeError):
        oracle.dense_attn(bad, q, K[:, :, :30], V[:, :, :30])
