"""Pins of the oracle's per-selection-set metadata scales (Sec. 3.2: the precision of the
compressed K cache may be traded; here every (sequence, KV head) - every sequence in joint
mode - stores its K_lr divided by a scale of its own), against things other than the oracle:
numpy brute force on the decoded values, a tensor library's float8 rounding, the identity
"a uniform array is the scalar", exactness of power-of-two scales, and a workload on which
one scale for all heads loses the selection that per-head scales keep."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import Shape

import brute


def _values():
    return np.array([oracle.fp8_e4m3_value(c) for c in range(256)])


def _inputs(seed, B=2, Hq=4, Hk=2, d=8, r=4, N=64):
    g = np.random.default_rng(seed)
    K = (g.standard_normal((B, Hk, N, d)) * 3).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.ascontiguousarray(g.standard_normal((Hk, d, r)).astype(np.float32))
    return K, q, A


@pytest.mark.parametrize("joint", [False, True])
def test_per_set_scales_match_brute_force_on_decoded_values(joint):
    B, Hq, Hk, d, r, N, G, M = 2, 4, 2, 8, 4, 64, 4, 5
    K, q, A = _inputs(11)
    mode = oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE
    scales = np.array([0.25, 1.5, 0.031, 7.0][: B if joint else B * Hk]).reshape((B,) if joint else (B, Hk))
    sh = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=oracle.FP8_E4M3, head_mode=mode, meta_scales=scales)
    klr, exact = oracle.build_metadata(sh, K, A, want_exact=True)
    ref_exact = (brute.joint_metadata(K.astype(np.float64), A.astype(np.float64)) if joint else
                 np.einsum("bknd,kdr->bknr", K.astype(np.float64), A.astype(np.float64)))
    np.testing.assert_allclose(exact, ref_exact, rtol=1e-13, atol=1e-14)     # exact = unscaled products
    sc = scales[..., None, None]                                            # one scale per set
    want = torch.from_numpy(np.clip(ref_exact / sc, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert (klr != want).mean() < 5e-3      # (the library rounds through fp32: rare ties differ)
    vals = _values()
    # every stored code is a nearest code of ITS set's scaled value
    xc = np.clip(ref_exact / sc, -448, 448)
    finite = np.array([c for c in range(256) if np.isfinite(vals[c])])
    best = np.abs(vals[finite][None, :] - xc.reshape(-1, 1)).min(1)
    np.testing.assert_allclose(np.abs(vals[klr].reshape(-1) - xc.reshape(-1)), best, rtol=0, atol=1e-12)
    deq = sc * vals[klr]
    res = oracle.predict_select(sh, q, klr, A)
    s_ref = (brute.joint_scores if joint else brute.scores)(q.astype(np.float64), deq, A.astype(np.float64))
    np.testing.assert_allclose(res["s"], s_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(res["idx"], brute.topk_groups(res["gs"], M))
    # a swapped pair of scales must change the stored codes (the index of the scale matters)
    swapped = scales.reshape(-1)[::-1].reshape(scales.shape)
    klr_sw = oracle.build_metadata(Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=oracle.FP8_E4M3, head_mode=mode,
                                         meta_scales=swapped), K, A)
    assert (klr_sw != klr).mean() > 0.5


@pytest.mark.parametrize("joint", [False, True])
@pytest.mark.parametrize("meta", [oracle.F32, oracle.BF16, oracle.FP8_E4M3])
def test_uniform_array_is_the_scalar(joint, meta):
    B, Hq, Hk, d, r, N, G, M = 2, 4, 2, 8, 4, 64, 4, 5
    K, q, A = _inputs(5)
    mode = oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE
    sets = (B,) if joint else (B, Hk)
    a = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=meta, head_mode=mode, meta_scale=0.37)
    b = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=meta, head_mode=mode, meta_scales=np.full(sets, 0.37))
    ka, kb = oracle.build_metadata(a, K, A), oracle.build_metadata(b, K, A)
    np.testing.assert_array_equal(ka, kb)
    ra, rb = oracle.predict_select(a, q, ka, A), oracle.predict_select(b, q, kb, A)
    np.testing.assert_array_equal(ra["idx"], rb["idx"])
    np.testing.assert_array_equal(ra["s"], rb["s"])


def test_power_of_two_scales_move_exponents_only():
    B, Hq, Hk, d, r, N, G, M = 2, 4, 2, 8, 4, 64, 4, 5
    K, q, A = _inputs(7)
    scales = np.array([[0.5, 4.0], [0.125, 16.0]])
    for meta in (oracle.F32, oracle.BF16):
        plain = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=meta)
        scaled = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=meta, meta_scales=scales)
        k1, k2 = oracle.build_metadata(plain, K, A), oracle.build_metadata(scaled, K, A)
        v = lambda k: k.astype(np.float64) if k.dtype == np.float32 else \
            (k.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        np.testing.assert_array_equal(v(k1), v(k2) * scales[..., None, None])
        np.testing.assert_array_equal(oracle.predict_select(plain, q, k1, A)["s"],
                                      oracle.predict_select(scaled, q, k2, A)["s"])


def test_bad_scales_are_rejected():
    K, q, A = _inputs(0)
    for bad in (np.array([[1.0, 0.0], [1.0, 1.0]]), np.array([[1.0, -2.0], [1.0, 1.0]]),
                np.array([[1.0, np.inf], [1.0, 1.0]])):
        with pytest.raises(RuntimeError):
            oracle.build_metadata(Shape(2, 4, 2, 8, 4, 64, 4, 5, meta_scales=bad), K, A)
    with pytest.raises(ValueError):
        Shape(2, 4, 2, 8, 4, 64, 4, 5, meta_scales=np.ones(3))


@pytest.mark.parametrize("ratio,one_scale_survives", [(2.0e3, True), (1.0e6, False)])
def test_per_head_scales_keep_the_selection_where_one_scale_loses_it(ratio, one_scale_survives):
    """Keys of one KV head `ratio` times larger than another's (heavy-hitter heads), 8-bit
    metadata.  An 8-bit FLOAT with one scale for all heads still ranks the small head's tokens
    at a ratio of 2000 (its values land between 2^-9 and 0.2, inside the format's range: this
    is why an integer format with per-row scales was not needed); at a ratio of 10^6 they fall
    below the smallest subnormal, all round to zero, and the selection degenerates to the
    first M groups.  A scale per head keeps both heads at any ratio."""
    B, Hq, Hk, d, r, N, G, M = 1, 4, 2, 16, 8, 512, 4, 16
    g = np.random.default_rng(21)
    K = g.standard_normal((B, Hk, N, d)).astype(np.float32)
    K[:, 0] *= np.float32(ratio ** 0.5)
    K[:, 1] *= np.float32(ratio ** -0.5)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.stack([np.linalg.qr(g.standard_normal((d, r)))[0] for _ in range(Hk)]).astype(np.float32)
    exact = Shape(B, Hq, Hk, d, r, N, G, M)                                      # fp32 metadata
    truth = oracle.predict_select(exact, q, oracle.build_metadata(exact, K, A), A)["idx"]
    absmax = np.abs(np.einsum("bknd,kdr->bknr", K.astype(np.float64), A.astype(np.float64))).max((2, 3))
    one = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=oracle.FP8_E4M3, meta_scale=float(absmax.max() / 400.0))
    per = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=oracle.FP8_E4M3, meta_scales=absmax / 400.0)
    recall = lambda sh: [len(set(a) & set(b)) / M for a, b in
                         zip(oracle.predict_select(sh, q, oracle.build_metadata(sh, K, A), A)["idx"][0], truth[0])]
    r_one, r_per = recall(one), recall(per)
    assert r_one[0] >= 0.7 and r_per[0] >= 0.7          # the large head is fine either way
    assert r_per[1] >= 0.7                              # the small head too with a scale of its own
    if one_scale_survives:
        assert r_one[1] >= 0.7
    else:
        assert r_one[1] <= 0.3                          # its metadata has vanished
