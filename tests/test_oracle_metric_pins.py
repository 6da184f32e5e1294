"""Pins for the oracle's tolerance ladder and ES_t / AS / fast_p (paper Sec. 3.4, App. D-F)."""
import math
import os

import numpy as np
import pytest

from oracle import metric

HERE = os.path.dirname(os.path.abspath(__file__))


def test_tolerances_reproduce_the_printed_table():
    for line in open(os.path.join(HERE, "golden", "tolerance_table.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        dt, a5, a0, r5, r0 = line[0], *map(float, line[1:])
        rt, at = metric.tolerance(dt, -5)
        assert at == pytest.approx(a5, rel=1e-12)
        assert rt == pytest.approx(r5, rel=0.04)          # the table prints two significant digits
        rt0, at0 = metric.tolerance(dt, 0)
        assert (rt0, at0) == (r0, a0)
    # log-linear: equal ratios between consecutive t
    for dt in ("bf16", "f32", "f64"):
        r = [metric.tolerance(dt, t) for t in range(-10, 1)]
        for k in range(1, 10):
            assert r[k][0] ** 2 == pytest.approx(r[k - 1][0] * r[k + 1][0], rel=1e-12)
            assert r[k][1] ** 2 == pytest.approx(r[k - 1][1] * r[k + 1][1], rel=1e-12)
        assert all(r[k][0] < r[k + 1][0] and r[k][1] < r[k + 1][1] for k in range(10))


def test_weights_and_their_sum():
    ts = range(-10, 5)
    assert [metric.weight(t) for t in (-10, -6, 4)] == [0.001] * 3
    assert [metric.weight(t) for t in (-5, -4, -3)] == [1.0] * 3
    assert metric.weight(-2) == pytest.approx(0.8) and metric.weight(3) == pytest.approx(0.8 ** 6)
    assert sum(metric.weight(t) for t in ts) == pytest.approx(5.957424, abs=1e-9)


def _case(speedup=1.0, error_class=0, pass_from=-10):
    """viol counts: zero from tolerance index pass_from upwards (11 = never passes)."""
    viol = [0 if t >= pass_from else 5 for t in metric.LADDER]
    return {"speedup": speedup, "error_class": error_class, "viol": viol}


def test_eager_row_scores_one():
    cases = [_case(1.0) for _ in range(7)]
    assert all(metric.es(cases, t) == pytest.approx(1.0) for t in range(-10, 5))
    assert metric.aggregated_score(cases) == pytest.approx(1.0)


def test_all_fail_floors():
    # every subgraph fails numerically at every t <= 0: ES_t = b for t < 1, 1 from t = 1 on
    acc = [_case(2.0, 0, pass_from=1) for _ in range(3)]
    assert metric.aggregated_score(acc) == pytest.approx(0.1 ** (4.957 / 5.957424), rel=1e-9)
    assert metric.aggregated_score(acc) == pytest.approx(0.14721, abs=1e-5)
    comp = [_case(2.0, 2) for _ in range(3)]
    assert metric.aggregated_score(comp) == pytest.approx(0.12565, abs=1e-5)
    run = [_case(2.0, 3) for _ in range(3)]
    assert metric.aggregated_score(run) == pytest.approx(0.11071, abs=1e-5)


def test_rectified_speedup_cases():
    ok_fast, ok_slow = _case(1.5), _case(0.5)
    assert metric.rectified_speedup(ok_fast, -5) == 1.5
    assert metric.rectified_speedup(ok_slow, -5, p=0.0) == 0.5
    assert metric.rectified_speedup(ok_slow, -5, p=0.5) == pytest.approx(0.5 ** 1.5)
    loose = _case(3.0, 0, pass_from=-3)                    # passes only from t = -3 on
    assert metric.rectified_speedup(loose, -4) == 0.1 and metric.rectified_speedup(loose, -3) == 3.0
    assert metric.rectified_speedup(loose, 2) == 3.0
    crash = _case(3.0, 3)
    assert [metric.rectified_speedup(crash, t) for t in (0, 2, 3, 4)] == [0.1, 0.1, 1.0, 1.0]


def test_es_equals_the_factored_form():
    # Prop. D.2: ES_t = alpha^lambda * beta^(lambda*eta*(p+1)) * gamma_t^(1-lambda)
    r = np.random.default_rng(0)
    b, p, t = 0.1, 0.3, 1
    cases = [_case(float(np.exp(r.normal(0, 0.5)))) for _ in range(11)] + [_case(1.0, 2), _case(1.0, 3), _case(2.0, 0, pass_from=1)]
    n = len(cases)
    good = [c for c in cases if metric.correct_at(c, t)]
    fast = [c["speedup"] for c in good if c["speedup"] >= 1]
    slow = [c["speedup"] for c in good if c["speedup"] < 1]
    lam, eta = len(good) / n, len(slow) / len(good)
    alpha = math.exp(sum(map(math.log, fast)) / len(good))
    beta = math.exp(sum(map(math.log, slow)) / len(slow))
    bad = [c for c in cases if not metric.correct_at(c, t)]
    cats = [c["error_class"] or 1 for c in bad]
    gamma = b ** (sum(1 for c in cats if t < c) / len(bad))
    want = alpha ** lam * beta ** (lam * eta * (p + 1)) * gamma ** (1 - lam)
    assert metric.es(cases, t, b, p) == pytest.approx(want, rel=1e-12)


def test_fast_p():
    cases = [_case(2.0), _case(1.05), _case(0.9), _case(3.0, 2), _case(3.0, 0, pass_from=-2)]
    assert metric.fast_p(cases, 1.0, t=0) == pytest.approx(3 / 5)
    assert metric.fast_p(cases, 1.0, t=-5) == pytest.approx(2 / 5)
    assert metric.fast_p(cases, 1.5, t=0) == pytest.approx(2 / 5)


def test_ladder_counts_are_monotone_and_hit_planted_levels():
    # elements with relative error 10^-k pass exactly from the level where rtol(t) reaches it
    b = np.ones(6, np.float32)
    a = (1.0 + np.array([0.0, 3e-7, 3e-5, 3e-3, 0.3, 30.0])).astype(np.float32)
    v = metric.ladder_violations(a, "f32", b, "f32")
    assert v == sorted(v, reverse=True) and v[-1] == 1 and v[0] == 5
    # f32 at t=-5: rtol 1.3e-6 + atol 1e-5 admits the 3e-7 error only
    assert v[5] == 4
