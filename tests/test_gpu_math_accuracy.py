"""Accuracy of the fp32 operators on their own: exp, tanh, sigmoid, gelu, division and rsqrt in fp32 graphs are
built from the hardware's one-ulp estimates with a correction step, not from correctly rounded library code.
Each is run as a one-operator subgraph over a dense sweep of arguments and compared with the fp64 oracle in
units in the last place of the exact result, together with the special values the definitions fix."""
import numpy as np
import pytest
import torch

from oracle import dag as oracle_dag
from tests.device import Runner, to_host_bits
from workloads import configs
from workloads.irtext import Builder

pytestmark = pytest.mark.gpu


def _unary(op, x, **attrs):
    g = Builder()
    g.output(g.op(op, [g.input("f32", x.shape)], "f32", **attrs))
    return configs.Workload(op, g.text(), [x], ["f32"], [x.shape], ["f32"], [x.shape]).finish()


def _ulps(got, ref):
    """|got - ref| in ulps of fp32 at ref (ref is the fp64 oracle value)."""
    r32 = ref.astype(np.float32)
    ulp = np.spacing(np.abs(r32)).astype(np.float64)
    ulp = np.maximum(ulp, 2.0 ** -149)
    return np.abs(got.astype(np.float64) - ref) / ulp


def _sweep(lo, hi, n=400000, seed=0):
    r = np.random.default_rng(seed)
    x = np.concatenate([np.linspace(lo, hi, n // 2), r.uniform(lo, hi, n // 2)]).astype(np.float32)
    return x.reshape(-1, 1000)


@pytest.mark.parametrize("op,lo,hi,bound", [("exp", -87.0, 88.0, 2.0), ("exp", -1.0, 1.0, 2.0), ("tanh", -9.5, 9.5, 3.5),
                                            ("tanh", -0.7, 0.7, 3.5), ("sigmoid", -80.0, 17.0, 3.0), ("rsqrt", 1e-6, 1e6, 2.0)])
def test_unary_operators_stay_within_a_few_ulp(op, lo, hi, bound):
    x = _sweep(lo, hi)
    w = _unary(op, x)
    out = Runner(w).run()[0]
    torch.cuda.synchronize()
    got = to_host_bits(out, "f32")
    ref = oracle_dag.run(w.text, w.inputs)[0]
    ok = np.abs(ref) > 1.2e-38                       # results below the normal range are flushed towards zero
    worst = float(_ulps(got[ok], ref[ok]).max())
    print(op, lo, hi, "worst ulp", worst, flush=True)
    assert worst <= bound, worst
    assert np.all(np.abs(got[~ok]) <= 1.2e-38)


def test_gelu_is_accurate_where_it_is_not_vanishing():
    x = _sweep(-4.0, 9.0)
    w = _unary("gelu", x, approx="tanh")
    got = to_host_bits(Runner(w).run()[0], "f32")
    ref = oracle_dag.run(w.text, w.inputs)[0]
    # far below zero the result is x * e^(2u) with 2u < -5: the fp32 rounding of u alone (|2u| * 1e-7, relative
    # to a vanishing result) is worth ten ulp and more there, whatever evaluates the exponential
    main = x >= -2.0
    worst = float(_ulps(got[main], ref[main]).max())
    print("gelu worst ulp for x >= -2:", worst, "worst abs error overall:", float(np.abs(got - ref).max()), flush=True)
    assert worst <= 8.0
    assert float(np.abs(got - ref).max()) <= 1e-6


def test_division_matches_the_definition_on_ordinary_and_special_operands():
    r = np.random.default_rng(3)
    a = (r.standard_normal(200000) * 10.0 ** r.uniform(-6, 6, 200000)).astype(np.float32)
    b = (r.standard_normal(200000) * 10.0 ** r.uniform(-6, 6, 200000)).astype(np.float32)
    special = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, np.nan, 1e-45, -3e-39, 1e-38, 3e38, -2.5e38, 1.7e38, 5e-324], np.float32)
    aa = np.concatenate([a, np.repeat(special, special.size)]).astype(np.float32)
    bb = np.concatenate([b, np.tile(special, special.size)]).astype(np.float32)
    pad = (-aa.size) % 8
    aa, bb = np.concatenate([aa, np.ones(pad, np.float32)]), np.concatenate([bb, np.ones(pad, np.float32)])
    g = Builder()
    g.output(g.op("div", [g.input("f32", aa.shape), g.input("f32", bb.shape)], "f32"))
    w = configs.Workload("div", g.text(), [aa, bb], ["f32", "f32"], [aa.shape] * 2, ["f32"], [aa.shape]).finish()
    got = to_host_bits(Runner(w).run()[0], "f32")
    with np.errstate(all="ignore"):
        ref = oracle_dag.run(w.text, w.inputs)[0]
        ref32 = ref.astype(np.float32)                 # the correctly rounded quotient, overflow and underflow included
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    inf = np.isinf(ref32)
    assert np.array_equal(got[inf], ref32[inf])
    zero = (ref32 == 0) & ~nan
    assert np.all(np.abs(got[zero]) <= 1.2e-38)
    rest = ~(nan | inf | zero) & (np.abs(ref) > 1.2e-38)
    assert float(_ulps(got[rest], ref[rest]).max()) <= 2.0
