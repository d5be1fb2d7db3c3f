"""Pins of the oracle's 8-bit metadata (Sec. 3.2: the precision of the compressed K cache
may be traded for memory; the format is the OCP 8-bit float E4M3, finite-only variant)
and of the metadata scale, against things other than itself."""
import numpy as np
import pytest
import torch

import oracle
from oracle import Shape
import brute


def _all_values():
    return np.array([oracle.fp8_e4m3_value(c) for c in range(256)])


def test_every_code_matches_the_float8_type_of_a_tensor_library():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = _all_values()
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    np.testing.assert_array_equal(got[~np.isnan(got)], ref[~np.isnan(ref)])


def test_hand_derived_code_values():
    v = oracle.fp8_e4m3_value
    assert v(0x00) == 0.0 and v(0x38) == 1.0 and v(0x3C) == 1.5          # bias 7: 0111.000 is 2^0
    assert v(0x7E) == 448.0 and v(0xFE) == -448.0                         # largest: 2^8 * 1.75
    assert v(0x08) == 2.0 ** -6 and v(0x01) == 2.0 ** -9 and v(0x07) == 7 * 2.0 ** -9   # subnormals
    assert np.isnan(v(0x7F)) and np.isnan(v(0xFF))


def test_rounding_hand_derived_ties_and_saturation():
    r = oracle.round_to_fp8_e4m3
    assert r(1.0) == 0x38
    assert r(1.0625) == 0x38      # halfway 1.0 / 1.125: even mantissa (000) wins
    assert r(1.1875) == 0x3A      # halfway 1.125 / 1.25: even mantissa (010) wins
    assert r(1.06250001) == 0x39
    assert r(464.0) == 0x7E and r(1e6) == 0x7E and r(-1e6) == 0xFE and r(448.0) == 0x7E   # saturates
    assert r(2.0 ** -10) == 0x00  # halfway 0 / smallest subnormal: even (0) wins
    assert r(1.5 * 2.0 ** -9) == 0x02   # halfway codes 1 and 2: even wins
    assert r(2.0 ** -10 * 1.0001) == 0x01
    assert r(-0.0) == 0x80 and r(0.0) == 0x00
    assert r(15.5) == 0x58        # 15.5 is halfway 15 (0x57, odd) / 16 (0x58, even)
    assert r(float("nan")) == 0x7F


def test_rounding_is_nearest_with_even_ties_by_search_over_all_codes():
    vals = _all_values()
    finite = np.where(~np.isnan(vals))[0]
    g = np.random.default_rng(0)
    xs = np.concatenate([g.standard_normal(2000) * s for s in (1e-3, 0.05, 1.0, 30.0, 300.0)])
    # exact midpoints between neighbouring positive values, too
    pos = np.sort(vals[finite][vals[finite] > 0])
    xs = np.concatenate([xs, (pos[:-1] + pos[1:]) / 2, -(pos[:-1] + pos[1:]) / 2])
    for x in xs:
        code = oracle.round_to_fp8_e4m3(float(x))
        xc = min(max(x, -448.0), 448.0)
        dist = np.abs(vals[finite] - xc)
        best = dist.min()
        assert abs(vals[code] - xc) == best, (x, code)
        ties = finite[dist == best]
        ties = [c for c in ties if (c & 0x80) == (code & 0x80) or vals[c] != 0]
        if len(ties) > 1 and x != 0:
            assert code & 1 == 0, (x, code, ties)        # even mantissa


def test_rounding_matches_the_tensor_library_in_range():
    g = np.random.default_rng(1)
    xs = np.concatenate([g.standard_normal(4000) * s for s in (0.01, 1.0, 100.0)])
    xs = xs[np.abs(xs) <= 448.0]
    ref = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.round_to_fp8_e4m3(float(x)) for x in xs], dtype=np.uint8)
    # the library converts through fp32 first; only values within fp32 rounding of a tie may differ
    assert (got != ref).mean() < 1e-3
    vals = _all_values()
    np.testing.assert_allclose(vals[got], vals[ref], rtol=0.13, atol=2.0 ** -9)


@pytest.mark.parametrize("joint", [False, True])
def test_whole_path_with_fp8_metadata_and_scale_matches_brute_force(joint):
    B, Hq, Hk, d, r, N, G, M = 2, 4, 2, 8, 4, 64, 4, 5
    g = np.random.default_rng(3)
    K = (g.standard_normal((B, Hk, N, d)) * 3).astype(np.float32)
    q = g.standard_normal((B, Hq, d)).astype(np.float32)
    A = np.ascontiguousarray(g.standard_normal((Hk, d, r)).astype(np.float32))
    scale = 0.25
    mode = oracle.HEADS_JOINT if joint else oracle.HEADS_SEPARATE
    sh = Shape(B, Hq, Hk, d, r, N, G, M, meta_dtype=oracle.FP8_E4M3, meta_scale=scale, head_mode=mode)
    klr, exact = oracle.build_metadata(sh, K, A, want_exact=True)
    assert klr.dtype == np.uint8
    ref_exact = (brute.joint_metadata(K.astype(np.float64), A.astype(np.float64)) if joint else
                 np.einsum("bknd,kdr->bknr", K.astype(np.float64), A.astype(np.float64)))
    np.testing.assert_allclose(exact, ref_exact, rtol=1e-13, atol=1e-14)      # exact = unscaled products
    # stored code = nearest code to exact / scale (library rounding, away from ties)
    want = torch.from_numpy(np.clip(ref_exact / scale, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert (klr != want).mean() < 5e-3
    vals = _all_values()
    deq = scale * vals[klr]
    res = oracle.predict_select(sh, q, klr, A)
    s_ref = (brute.joint_scores if joint else brute.scores)(q.astype(np.float64), deq, A.astype(np.float64))
    np.testing.assert_allclose(res["s"], s_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(res["idx"], brute.topk_groups(res["gs"], M))
    # a power-of-two scale moves exponents only: bf16/fp32 metadata scaled and unscaled agree exactly
    sh1 = Shape(B, Hq, Hk, d, r, N, G, M, head_mode=mode)
    sh2 = Shape(B, Hq, Hk, d, r, N, G, M, head_mode=mode, meta_scale=4.0)
    k1, k2 = oracle.build_metadata(sh1, K, A), oracle.build_metadata(sh2, K, A)
    np.testing.assert_array_equal(k1, k2 * np.float32(4.0))
    np.testing.assert_array_equal(oracle.predict_select(sh1, q, k1, A)["s"],
                                  oracle.predict_select(sh2, q, k2, A)["s"])


def test_bad_scale_is_rejected():
    g = np.random.default_rng(0)
    K = g.standard_normal((1, 1, 8, 8)).astype(np.float32)
    A = np.ascontiguousarray(g.standard_normal((1, 8, 4)).astype(np.float32))
    with pytest.raises(RuntimeError):
        oracle.build_metadata(Shape(1, 1, 1, 8, 4, 8, 4, 1, meta_scale=-1.0), K, A)
    with pytest.raises(RuntimeError):
        oracle.build_metadata(Shape(1, 1, 1, 8, 4, 8, 4, 1, kv_dtype=oracle.FP8_E4M3), K.view(np.uint8)[..., :8], A)
