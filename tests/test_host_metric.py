"""Host-only tests of the library's tolerance ladder and ES_t / AS / fast_p against the oracle."""
import numpy as np
import pytest

import paper_2605_29357_amd as pf
from oracle import metric


def test_tolerances_equal_the_oracle_bit_for_bit():
    for dt in ("bf16", "f32", "f64"):
        for t in range(-10, 5):
            assert pf.tolerance(dt, t) == metric.tolerance(dt, t)


def _random_cases(seed, n):
    r = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        kind = r.integers(0, 5)
        pass_from = int(r.integers(-10, 2))          # 1: never passes numerically
        viol = [0 if t >= pass_from else int(r.integers(1, 1000)) for t in metric.LADDER]
        cases.append({"speedup": float(np.exp(r.normal(0.1, 0.6))), "error_class": [0, 0, 0, 2, 3][kind], "viol": viol})
    return cases


@pytest.mark.parametrize("b,p", [(0.1, 0.0), (0.3, 0.5)])
def test_es_and_as_match_the_oracle(b, p):
    for seed in range(5):
        cases = _random_cases(seed, 1 + 7 * seed)
        es, a = pf.aggregate(cases, b, p)
        for k, t in enumerate(range(-10, 5)):
            assert es[k] == pytest.approx(metric.es(cases, t, b, p), rel=1e-13)
        assert a == pytest.approx(metric.aggregated_score(cases, b, p), rel=1e-13)
        for t in (-5, 0, 3):
            assert pf.fast_p(cases, 1.0, t) == metric.fast_p(cases, 1.0, t)


def test_reference_execution_scores_one_and_floors():
    ok = [{"speedup": 1.0, "error_class": 0, "viol": [0] * 11}] * 4
    es, a = pf.aggregate(ok)
    assert all(abs(e - 1) < 1e-15 for e in es) and abs(a - 1) < 1e-15
    bad = [{"speedup": 2.0, "error_class": 0, "viol": [3] * 11}] * 4
    assert pf.aggregate(bad)[1] == pytest.approx(0.14721, abs=1e-5)


def test_bad_cases_are_refused():
    with pytest.raises(pf.PfError):
        pf.aggregate([{"speedup": 1.0, "error_class": 1, "viol": [0] * 11}])
    with pytest.raises(pf.PfError):
        pf.aggregate([{"speedup": -1.0, "error_class": 0, "viol": [0] * 11}])
