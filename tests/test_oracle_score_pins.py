"""Pins for the oracle's error scorer (paper Eq. 1 with atol/rtol of Appendix F)."""
import numpy as np
import pytest

from oracle.score import score_pair


def f32(a):
    return np.asarray(a, dtype=np.float32)


def test_identical_buffers_score_zero():
    x = f32(np.random.default_rng(0).normal(size=1000))
    r = score_pair(x, "f32", x.copy(), "f32", 0.0, 0.0)
    assert r["max_abs"] == 0 and r["max_rel"] == 0 and r["n_viol"] == 0
    assert r["allclose"] == 1 and r["bit_identical"] == 1 and r["n"] == 1000


def test_planted_outlier_of_known_size():
    b = np.ones(1000, np.float32) * 2
    a = b.copy()
    a[123] = 2.5
    r = score_pair(a, "f32", b, "f32", rtol=0.1, atol=0.0)
    assert r["max_abs"] == 0.5 and r["max_rel"] == 0.25
    assert r["n_viol"] == 1 and r["allclose"] == 0 and r["bit_identical"] == 0
    r = score_pair(a, "f32", b, "f32", rtol=0.25, atol=0.0)          # boundary is inclusive
    assert r["n_viol"] == 0 and r["allclose"] == 1
    r = score_pair(a, "f32", b, "f32", rtol=0.0, atol=0.5)
    assert r["n_viol"] == 0


def test_tolerance_scales_with_the_reference_not_the_candidate():
    # |1 - 2| = 1 <= 0.5 * |ref|: true for ref = 2, false for ref = 1
    assert score_pair(f32([1]), "f32", f32([2]), "f32", 0.5, 0.0)["allclose"] == 1
    assert score_pair(f32([2]), "f32", f32([1]), "f32", 0.5, 0.0)["allclose"] == 0


def test_nan_and_inf_counts_and_their_treatment():
    b = f32([1, 2, np.inf, -np.inf, np.nan, 0, 0, 5])
    a = f32([1, np.nan, np.inf, np.inf, np.nan, 0, 1e-3, np.inf])
    r = score_pair(a, "f32", b, "f32", rtol=1e-2, atol=1e-2)
    assert (r["nan_cand"], r["nan_ref"], r["inf_cand"], r["inf_ref"]) == (2, 1, 3, 2)
    # violations: NaN vs 2, +inf vs -inf, NaN vs NaN (equal_nan off), +inf vs 5
    assert r["n_viol"] == 4 and r["allclose"] == 0
    assert r["max_abs"] == np.inf and r["max_rel"] == np.inf
    r2 = score_pair(a, "f32", b, "f32", rtol=1e-2, atol=1e-2, equal_nan=True)
    assert r2["n_viol"] == 3
    # equal infinities are close and contribute zero error
    r3 = score_pair(f32([np.inf, 1]), "f32", f32([np.inf, 1]), "f32", 0, 0)
    assert r3["allclose"] == 1 and r3["max_abs"] == 0 and r3["inf_cand"] == 1


def test_relative_error_with_zero_reference():
    r = score_pair(f32([0, 1e-3]), "f32", f32([0, 0]), "f32", 1e-2, 1e-2)
    assert r["max_rel"] == np.inf and r["max_abs"] == float(np.float32(1e-3)) and r["allclose"] == 1
    r = score_pair(f32([0, 0]), "f32", f32([0, 0]), "f32", 0, 0)
    assert r["max_rel"] == 0


@pytest.mark.parametrize("rtol,atol", [(1e-5, 1e-5), (2e-2, 1e-5), (0.0, 1e-3), (1e-3, 0.0)])
def test_violation_count_matches_numpy_isclose(rtol, atol):
    # numpy.isclose is the same asymmetric test |a-b| <= atol + rtol*|b|
    rng = np.random.default_rng(7)
    b = rng.normal(size=5000).astype(np.float32)
    a = (b.astype(np.float64) * (1 + rng.normal(size=5000) * rtol) + rng.normal(size=5000) * atol).astype(np.float32)
    r = score_pair(a, "f32", b, "f32", rtol, atol)
    want = np.isclose(a.astype(np.float64), b.astype(np.float64), rtol=rtol, atol=atol)
    assert r["n_viol"] == int((~want).sum())
    assert 0 < r["n_viol"] < 5000
    d = np.abs(a.astype(np.float64) - b.astype(np.float64))
    assert r["max_abs"] == d.max()


def test_mixed_dtypes_widen_exactly():
    # bf16 0x3F81 = 1.0078125; fp64 reference a hair away
    r = score_pair(np.array([0x3F81], np.uint16), "bf16", np.array([1.0], np.float64), "f64", 0, 0)
    assert r["max_abs"] == 0.0078125 and r["bit_identical"] == 0
    r = score_pair(np.array([0x3F81, 0x7FC0], np.uint16), "bf16", np.array([0x3F81, 0x7FC0], np.uint16), "bf16", 0, 0)
    assert r["bit_identical"] == 1 and r["allclose"] == 0 and r["nan_cand"] == 1


def test_signed_zeros_compare_equal_but_differ_in_bits():
    r = score_pair(f32([0.0]), "f32", f32([-0.0]), "f32", 0, 0)
    assert r["allclose"] == 1 and r["max_abs"] == 0 and r["bit_identical"] == 0


def test_empty_pair():
    r = score_pair(f32([]), "f32", f32([]), "f32", 0, 0)
    assert r["n"] == 0 and r["allclose"] == 1 and r["max_abs"] == 0 and r["bit_identical"] == 1


def test_fp16_pairs_are_scored_on_the_widened_values():
    # 0x4000 = 2.0, 0x4001 = 2 + 2^-9, 0x3C00 = 1.0, 0x7C00 = inf, 0x7E00 = NaN
    cand = np.array([0x3C00, 0x4001, 0x3C00, 0x7C00, 0x7E00, 0x0001], np.uint16)
    ref = np.array([0x3C00, 0x4000, 0xBC00, 0x7C00, 0x3C00, 0x0000], np.uint16)
    r = score_pair(cand, "f16", ref, "f16", rtol=1e-3, atol=1e-5)
    assert r["n"] == 6 and r["nan_cand"] == 1 and r["nan_ref"] == 0 and r["inf_cand"] == 1 and r["inf_ref"] == 1
    assert r["max_abs"] == 2.0                      # 1 vs -1; the NaN element is left out of the maxima
    assert r["max_rel"] == np.inf                   # 2^-24 against a zero reference
    # violations: 2+2^-9 vs 2 (0.00195 > 1e-5 + 2e-3? no: allowed 0.00201) passes; 1 vs -1 fails; NaN fails;
    # 2^-24 vs 0 passes on atol; equal infinities pass
    assert r["n_viol"] == 2 and r["allclose"] == 0 and r["bit_identical"] == 0
    same = score_pair(ref, "f16", ref, "f16", rtol=0.0, atol=0.0)
    assert same["allclose"] == 1 and same["bit_identical"] == 1 and same["max_abs"] == 0.0
    mixed = score_pair(np.array([0x4001], np.uint16), "f16", np.array([2.0], np.float32), "f32", rtol=0.0, atol=2.0 ** -9)
    assert mixed["max_abs"] == 2.0 ** -9 and mixed["allclose"] == 1
