"""CPU oracle: error scoring of a (candidate, reference) output pair in fp64.

TEST INFRASTRUCTURE ONLY; the product path never imports this.

A rewrite is valid when the error between the reference and the rewritten
subgraph's outputs stays within a tolerance (paper Eq. 1).  The paper does not
define err(.,.); it only names atol(t) and rtol(t) (Appendix F).  The reading
used here is the asymmetric element-wise test
        a == b   or   ( |a - b| is finite and |a - b| <= atol + rtol * |b| )
with b the reference.  NaNs never pass unless equal_nan is set and both sides
are NaN at that element.  Besides the pass/fail count the scorer reports the
largest absolute and relative error over the elements where neither side is
NaN, NaN/Inf counts per side, and whether the two buffers hold the same bits.

relative error of one element: 0 if a == b; +inf if b == 0 or |a - b| is
infinite; otherwise |a - b| / |b|.
"""
import numpy as np

from .dag import upconvert


def score_pair(cand, cand_dtype, ref, ref_dtype, rtol, atol, equal_nan=False):
    """cand/ref: stored arrays ('f32' float32, 'bf16' / 'f16' uint16 bits, 'f64' float64)."""
    a = _widen(cand, cand_dtype).ravel()
    b = _widen(ref, ref_dtype).ravel()
    if a.size != b.size:
        raise ValueError("size mismatch")
    n = a.size
    nan_a, nan_b = np.isnan(a), np.isnan(b)
    res = {
        "n": int(n),
        "nan_cand": int(nan_a.sum()), "nan_ref": int(nan_b.sum()),
        "inf_cand": int(np.isinf(a).sum()), "inf_ref": int(np.isinf(b).sum()),
    }
    anynan = nan_a | nan_b
    both_nan = nan_a & nan_b
    ok = ~anynan
    with np.errstate(all="ignore"):
        eq = a == b
        d = np.where(eq, 0.0, np.abs(a - b))
        absb = np.abs(b)
        rel = np.where(eq, 0.0, np.where((b == 0.0) | np.isinf(d), np.inf, d / absb))
        allowed = atol + rtol * absb
        close = eq | (np.isfinite(d) & (d <= allowed))
    close = np.where(anynan, both_nan if equal_nan else False, close)
    res["max_abs"] = float(d[ok].max()) if ok.any() else 0.0
    res["max_rel"] = float(rel[ok].max()) if ok.any() else 0.0
    res["n_viol"] = int(n - int(np.count_nonzero(close)))
    res["allclose"] = int(res["n_viol"] == 0)
    if cand_dtype == ref_dtype:
        res["bit_identical"] = int(np.array_equal(_bits(cand, cand_dtype), _bits(ref, ref_dtype)))
    else:
        res["bit_identical"] = 0
    return res


def _widen(x, dtype):
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    return upconvert(x, dtype)


def _bits(x, dtype):
    x = np.ascontiguousarray(x)
    if dtype == "f32":
        return x.view(np.uint32).ravel()
    if dtype == "f64":
        return x.view(np.uint64).ravel()
    return x.view(np.uint16).ravel()
