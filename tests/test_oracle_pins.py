"""Pins for the CPU oracle: closed forms, invariants, brute force, library routines.

None of these call the HIP library.  Each pin is chosen so that a plausible
slip in oracle/dag.py (dropped term, wrong sign or index, transposed operand,
biased/unbiased variance, eps outside the root, wrong broadcast axis) fails it.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import dag
from workloads import configs, rng
from workloads.irtext import Builder


def run1(text, inputs):
    return dag.run(text, inputs)[0]


def f32(a):
    return np.asarray(a, dtype=np.float32)


# ---------------------------------------------------------------- LayerNorm
def _ln_workload(rows=8, cols=96, seed=11, unit_affine=True, **kw):
    w = configs.cfg1_add_layernorm(rows=rows, cols=cols, seed=seed, **kw)
    if unit_affine:
        w.inputs[2] = np.ones(cols, np.float32)
        w.inputs[3] = np.zeros(cols, np.float32)
    return w


@pytest.mark.parametrize("use_var_op", [False, True])
def test_layernorm_zero_mean_and_closed_form_variance(use_var_op):
    # Before the affine step a LayerNorm row has mean 0 and variance v/(v+eps),
    # v the biased variance of the row (paper Case 1: divide by C, eps inside rsqrt).
    w = _ln_workload(use_var_op=use_var_op)
    y = run1(w.text, w.inputs)
    h = w.inputs[0].astype(np.float64) + w.inputs[1].astype(np.float64)
    v = h.var(axis=-1)                       # numpy's biased variance: library routine
    assert np.abs(y.mean(axis=-1)).max() < 1e-13
    np.testing.assert_allclose(y.var(axis=-1), v / (v + 1e-5), rtol=1e-12)
    # an unbiased variance or eps outside the root would miss this by > 1e-3 / 1e-6
    assert np.abs(y.var(axis=-1) - 1.0).max() < 1e-4


def test_layernorm_hand_row():
    # h = [1,2,3,4] + 0: mean 2.5, biased variance 1.25
    w = _ln_workload(rows=1, cols=4)
    w.inputs[0] = f32([[1, 2, 3, 4]])
    w.inputs[1] = f32([[0, 0, 0, 0]])
    w.inputs[2] = f32([2, 2, 2, 2])
    w.inputs[3] = f32([0.5, 0.5, 0.5, 0.5])
    s = math.sqrt(1.25 + 1e-5)
    want = [2 * d / s + 0.5 for d in (-1.5, -0.5, 0.5, 1.5)]
    np.testing.assert_allclose(run1(w.text, w.inputs)[0], want, rtol=1e-14)


def test_layernorm_shift_invariance_and_affine():
    w = _ln_workload(unit_affine=False)
    y0 = run1(w.text, w.inputs)
    w2 = _ln_workload(unit_affine=False)
    w2.inputs[1] = w2.inputs[1] + np.float32(4.0)         # exact in fp32 for |r| < 2^20
    # adding a constant to every element of the row changes nothing
    np.testing.assert_allclose(run1(w2.text, w2.inputs), y0, rtol=0, atol=2e-6)
    # affine step: y = yhat * gamma + beta, gamma and beta indexed by column
    w1 = _ln_workload(unit_affine=True)
    yhat = run1(w1.text, w1.inputs)
    g, b = w.inputs[2].astype(np.float64), w.inputs[3].astype(np.float64)
    np.testing.assert_allclose(y0, yhat * g[None, :] + b[None, :], rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ softmax
def test_softmax_rows_sum_to_one_and_mask_is_exact():
    w = configs.cfg2_masked_softmax(heads=2, seq=64, seed=5)
    y = run1(w.text, w.inputs)
    assert np.abs(y.sum(axis=-1) - 1.0).max() < 1e-14
    assert y.min() >= 0.0 and y.max() <= 1.0
    iu = np.triu_indices(64, k=1)
    assert (y[:, iu[0], iu[1]] == 0.0).all()              # masked entries are exactly zero
    assert (y[:, 0, 0] == 1.0).all()                       # row 0 keeps only its diagonal
    il = np.tril_indices(64)
    assert (y[:, il[0], il[1]] > 0.0).all()


def test_softmax_constant_logits_closed_form():
    # equal logits: row i is 1/(i+1) on its first i+1 entries
    w = configs.cfg2_masked_softmax(heads=1, seq=32, seed=5)
    w.inputs[0] = np.full((1, 32, 32), 0x4040, np.uint16)   # bf16 3.0
    y = run1(w.text, w.inputs)[0]
    for i in range(32):
        np.testing.assert_allclose(y[i, :i + 1], 1.0 / (i + 1), rtol=1e-15)
        assert (y[i, i + 1:] == 0).all()


def test_softmax_against_direct_formula_and_scale():
    # two unmasked logits: softmax = logistic of the scaled difference
    g = Builder()
    z = g.input("f32", (1, 2))
    m = g.input("f32", (1, 2))
    s = g.const(0.125, "f32")
    t = g.op("add", [g.op("mul", [z, s], "f32"), m], "f32")
    e = g.op("exp", [g.op("sub", [t, g.op("max", [t], "f32")], "f32")], "f32")
    g.output(g.op("div", [e, g.op("sum", [e], "f32")], "f32"))
    y = run1(g.text(), [f32([[8.0, -8.0]]), f32([[0, 0]])])
    want = 1.0 / (1.0 + math.exp(-2.0))                   # (8 - -8) * 0.125 = 2
    np.testing.assert_allclose(y[0], [want, 1 - want], rtol=1e-14)


def test_softmax_fully_masked_row_is_nan():
    w = configs.cfg2_masked_softmax(heads=1, seq=4, seed=5)
    w.inputs[1][:] = 0xFF80
    assert np.isnan(run1(w.text, w.inputs)).all()


# --------------------------------------------------------------------- GELU
def _unary(op, x, **attrs):
    g = Builder()
    i = g.input("f32", (len(x),))
    g.output(g.op(op, [i], "f32", **attrs))
    return run1(g.text(), [f32(x)])


def test_gelu_tanh_identities_and_closeness_to_exact():
    x = np.linspace(-6, 6, 241).astype(np.float32)
    y = _unary("gelu", x, approx="tanh")
    ym = _unary("gelu", -x, approx="tanh")
    assert _unary("gelu", [0.0], approx="tanh")[0] == 0.0
    np.testing.assert_allclose(y - ym, x.astype(np.float64), rtol=0, atol=1e-15)   # gelu(x)-gelu(-x)=x
    # exact GELU is x * Phi(x); the tanh form stays within 5e-4 of it (wrong
    # sqrt(2/pi) or 0.044715 moves it by more)
    exact = np.array([v * 0.5 * (1 + math.erf(v / math.sqrt(2))) for v in x.astype(np.float64)])
    assert np.abs(y - exact).max() < 5e-4
    assert np.abs(y - exact).max() > 1e-5                 # and is not the erf form itself
    # tails
    assert abs(_unary("gelu", [10.0], approx="tanh")[0] - 10.0) < 1e-12
    assert abs(_unary("gelu", [-10.0], approx="tanh")[0]) < 1e-12


def test_gelu_erf_is_x_times_normal_cdf():
    from scipy.stats import norm
    x = np.linspace(-5, 5, 101).astype(np.float32)
    y = _unary("gelu", x, approx="erf")
    np.testing.assert_allclose(y, x.astype(np.float64) * norm.cdf(x.astype(np.float64)), rtol=1e-12, atol=1e-15)


def test_gelu_gate_bias_broadcasts_along_columns():
    w = configs.cfg3_bias_gelu_gate(rows=3, cols=8, seed=9)
    w.inputs[0][:] = 0                                   # a = 0 -> argument is the bias alone
    w.inputs[2][:] = 0x3F80                              # b = 1
    y = run1(w.text, w.inputs)
    bias = dag.upconvert(w.inputs[1], "bf16")
    col = np.array([0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3))) for v in bias])
    for r in range(3):
        np.testing.assert_allclose(y[r], col, rtol=1e-14, atol=0)
    assert len(set(np.round(col, 12))) > 1               # the columns do differ


# ---------------------------------------------------- other unary operators
def test_unary_ops_against_libm_and_identities():
    x = np.linspace(-4, 4, 33).astype(np.float32)
    xd = x.astype(np.float64)
    np.testing.assert_allclose(_unary("exp", x), [math.exp(v) for v in xd], rtol=1e-15)
    np.testing.assert_allclose(_unary("tanh", x), [math.tanh(v) for v in xd], rtol=1e-15, atol=1e-300)
    s = _unary("sigmoid", x)
    np.testing.assert_allclose(s + _unary("sigmoid", -x), 1.0, rtol=1e-15)      # s(x)+s(-x)=1
    np.testing.assert_allclose(s, 0.5 * (1 + np.tanh(xd / 2)), rtol=1e-14)      # textbook identity
    p = np.array([0.25, 1.0, 4.0, 16.0], np.float32)
    np.testing.assert_array_equal(_unary("rsqrt", p), [2.0, 1.0, 0.5, 0.25])


# ----------------------------------------------------------- RMSNorm + RoPE
def _rope(batch=1, positions=8, heads=2, dim=16, seed=21):
    return configs.cfg4_rmsnorm_rope(batch=batch, positions=positions, heads=heads, dim=dim, seed=seed)


def test_rmsnorm_unit_weight_closed_form_and_position_zero():
    w = _rope()
    w.inputs[1][:] = 0x3F80                              # weight = 1
    y = run1(w.text, w.inputs)
    x = dag.upconvert(w.inputs[0], "bf16")
    ms = (x * x).mean(axis=-1)
    # rotation preserves the norm of each pair, hence mean(y^2) = ms/(ms+eps)
    # (to the fp32 rounding of the tables: cos^2 + sin^2 = 1 +- 2^-23)
    np.testing.assert_allclose((y * y).mean(axis=-1), ms / (ms + 1e-6), rtol=3e-7)
    assert np.abs((y * y).mean(axis=-1) - 1.0).max() < 1e-5
    # position 0 turns by angle 0: output is the plain RMSNorm
    np.testing.assert_allclose(y[:, 0], x[:, 0] / np.sqrt(ms[:, 0] + 1e-6)[..., None], rtol=1e-13)


def test_rmsnorm_weight_is_per_column_plain_factor():
    w = _rope()
    y = run1(w.text, w.inputs)
    w1 = _rope()
    w1.inputs[1][:] = 0x3F80
    y1 = run1(w1.text, w1.inputs)
    wt = dag.upconvert(w.inputs[1], "bf16")
    # at position 0 (no rotation) the weight multiplies column-wise: y = y1 * w, not (1 + w)
    np.testing.assert_allclose(y[:, 0], y1[:, 0] * wt, rtol=1e-13)


def test_rotary_angles_direction_and_inverse():
    pos, dim = 8, 16
    cos, sin = configs.rotary_tables(pos, dim)
    # theta(p, i) = p * 10000^(-2i/dim): pair 0 turns by p radians
    np.testing.assert_allclose(cos[:, 0, 0], np.cos(np.arange(pos)), atol=1e-7)
    np.testing.assert_allclose(sin[:, 0, 1], np.sin(np.arange(pos)), atol=1e-7)
    np.testing.assert_allclose(cos[1, 0, 2], math.cos(10000 ** (-2 / 16)), atol=1e-7)
    full_c, _ = configs.rotary_tables(2048, 128)
    assert abs(math.acos(full_c[1, 0, 2]) - 0.8659643233600653) < 1e-6
    assert abs(math.acos(full_c[1000, 0, 126]) / 1000 - 1.1547819846894582e-4) < 1e-8
    # y = n*cos + rot_pairs(n)*sin on a pair (1, 0) gives (cos, sin): a counter-clockwise turn
    g = Builder()
    n = g.input("f32", (pos, 1, dim))
    c = g.input("f32", (pos, 1, dim))
    s = g.input("f32", (pos, 1, dim))
    g.output(g.op("add", [g.op("mul", [n, c], "f32"),
                          g.op("mul", [g.op("rot_pairs", [n], "f32"), s], "f32")], "f32"))
    e = np.zeros((pos, 1, dim), np.float32)
    e[..., 0::2] = 1.0
    y = run1(g.text(), [e, cos, sin])
    np.testing.assert_array_equal(y[..., 0::2], cos[..., 0::2].astype(np.float64))
    np.testing.assert_array_equal(y[..., 1::2], sin[..., 1::2].astype(np.float64))
    # turning by theta and then by -theta is the identity
    v = f32(np.random.default_rng(0).normal(size=(pos, 1, dim)))
    back = run1(g.text(), [run1(g.text(), [v, cos, sin]).astype(np.float32), cos, -sin])
    np.testing.assert_allclose(back, v, atol=1e-6)


def test_rot_pairs_definition():
    g = Builder()
    i = g.input("f32", (2, 6))
    g.output(g.op("rot_pairs", [i], "f32"))
    x = f32([[1, 2, 3, 4, 5, 6], [7, 8, 9, 10, 11, 12]])
    np.testing.assert_array_equal(run1(g.text(), [x]), [[-2, 1, -4, 3, -6, 5], [-8, 7, -10, 9, -12, 11]])


# ---------------------------------------- elementwise / broadcast / movement
def _brute_binary(op, a, b):
    """Right-aligned broadcasting by explicit index arithmetic (pure Python)."""
    ra, rb = a.ndim, b.ndim
    r = max(ra, rb)
    sa = (1,) * (r - ra) + a.shape
    sb = (1,) * (r - rb) + b.shape
    so = tuple(max(x, y) for x, y in zip(sa, sb))
    a2, b2 = a.reshape(sa), b.reshape(sb)
    out = np.empty(so, np.float64)
    for idx in itertools.product(*[range(d) for d in so]):
        ia = tuple(i if d > 1 else 0 for i, d in zip(idx, sa))
        ib = tuple(i if d > 1 else 0 for i, d in zip(idx, sb))
        x, y = float(a2[ia]), float(b2[ib])
        out[idx] = {"add": x + y, "sub": x - y, "mul": x * y, "div": x / y}[op]
    return out


@pytest.mark.parametrize("op", ["add", "sub", "mul", "div"])
@pytest.mark.parametrize("shapes", [((2, 3, 4), (4,)), ((2, 3, 4), (3, 1)), ((2, 3, 4), (2, 1, 4)),
                                    ((3, 1), (2, 1, 4)), ((4,), (2, 3, 4)), ((2, 3, 4), (2, 3, 4))])
def test_binary_broadcast_brute_force(op, shapes):
    r = np.random.default_rng(3)
    a = f32(r.uniform(1, 2, size=shapes[0]))
    b = f32(r.uniform(1, 2, size=shapes[1]))
    g = Builder()
    ia = g.input("f32", shapes[0])
    ib = g.input("f32", shapes[1])
    g.output(g.op(op, [ia, ib], "f32"))
    np.testing.assert_array_equal(run1(g.text(), [a, b]), _brute_binary(op, a, b))


def test_const_and_operand_order():
    g = Builder()
    i = g.input("f32", (3,))
    c = g.const(10.0, "f32")
    g.output(g.op("sub", [c, i], "f32"))
    g.output(g.op("div", [i, c], "f32"))
    y = dag.run(g.text(), [f32([1, 2, 4])])
    np.testing.assert_array_equal(y[0], [9, 8, 6])
    np.testing.assert_array_equal(y[1], [0.1, 0.2, 0.4])


def test_transpose_is_an_involution_and_moves_the_right_axes():
    g = Builder()
    i = g.input("f32", (2, 3, 5))
    t = g.op("transpose", [i], "f32")
    g.output(t)
    g.output(g.op("transpose", [t], "f32"))
    x = f32(np.arange(30).reshape(2, 3, 5))
    y = dag.run(g.text(), [x])
    assert y[0].shape == (2, 5, 3)
    for b, r, c in itertools.product(range(2), range(3), range(5)):
        assert y[0][b, c, r] == x[b, r, c]
    np.testing.assert_array_equal(y[1], x)


# --------------------------------------------------------------- reductions
def _reduce(op, x, **attrs):
    g = Builder()
    i = g.input("f32", x.shape)
    g.output(g.op(op, [i], "f32", **attrs))
    return run1(g.text(), [x])


def test_reductions_closed_forms():
    ones = np.ones((3, 7), np.float32)
    assert _reduce("sum", ones).shape == (3, 1)
    assert _reduce("sum", ones, keepdim=0).shape == (3,)
    np.testing.assert_array_equal(_reduce("sum", ones), 7.0)
    np.testing.assert_array_equal(_reduce("mean", 3 * ones), 3.0)
    x = f32([[1, 2, 3, 4], [4, 4, 4, 4]])
    np.testing.assert_array_equal(_reduce("var", x), [[1.25], [0.0]])
    np.testing.assert_allclose(_reduce("var", x, correction=1), [[5.0 / 3.0], [0.0]], rtol=1e-15)
    np.testing.assert_array_equal(_reduce("sum", x), [[10], [16]])        # rows, not columns
    p = np.zeros((2, 9), np.float32)
    p[1, 5] = 7.5
    p[0, :] = -3
    np.testing.assert_array_equal(_reduce("max", p), [[-3], [7.5]])
    q = p.copy()
    q[0, 2] = np.nan
    m = _reduce("max", q)
    assert np.isnan(m[0, 0]) and m[1, 0] == 7.5


def test_reduction_over_last_dim_of_rank3_matches_numpy():
    x = f32(np.random.default_rng(1).normal(size=(2, 3, 17)))
    xd = x.astype(np.float64)
    np.testing.assert_allclose(_reduce("sum", x)[..., 0], xd.sum(-1), rtol=1e-14)
    np.testing.assert_allclose(_reduce("mean", x)[..., 0], xd.mean(-1), rtol=1e-14, atol=1e-16)
    np.testing.assert_array_equal(_reduce("max", x)[..., 0], xd.max(-1))
    np.testing.assert_allclose(_reduce("var", x)[..., 0], xd.var(-1), rtol=1e-13)


# --------------------------------------------------------------- IR reading
def test_inputs_are_widened_exactly_and_never_rounded():
    # bf16 1.0078125 = 0x3F81; (x * x) keeps bits a bf16 or fp32 result would drop
    g = Builder()
    i = g.input("bf16", (1,))
    m = g.op("mul", [i, i], "bf16")
    g.output(g.op("mul", [m, m], "bf16"))
    y = run1(g.text(), [np.array([0x3F81], np.uint16)])
    sq = 1.0078125 * 1.0078125                      # 15 significant bits: exact in fp64, not in bf16
    assert y[0] == sq * sq                           # 29 bits: exact in fp64, not in fp32


def test_parser_rejects_bad_text():
    for bad in ["in %1 : f32[2]\n", "in %0 : f32[2]\n%1 = add(%0, %2) : f32\n", "garbage\n"]:
        with pytest.raises(ValueError):
            dag.parse(bad)


def test_f32_mode_is_the_same_definition_in_single_precision():
    w = _ln_workload()
    y64 = run1(w.text, w.inputs)
    y32 = dag.run(w.text, w.inputs, dtype=np.float32)[0]
    assert y32.dtype == np.float32
    np.testing.assert_allclose(y32, y64, rtol=1e-5, atol=1e-5)


# ------------------------------------------------------------- roll and slice
def _view_graph(shape, steps):
    g = Builder()
    t = g.input("f32", shape)
    for op, attrs in steps:
        t = g.op(op, [t], "f32", **attrs)
    g.output(t)
    return g.text()


def test_roll_then_prefix_slice_is_the_index_formula_of_case_1():
    # out[i, j, :] = x[(S + i - shift) mod S, (S + j - shift) mod S, :] for i, j < SC
    S, SC, C, shift = 7, 5, 3, 3
    x = f32(np.arange(S * S * C).reshape(S, S, C))
    text = _view_graph((S, S, C), [("roll", dict(shift=shift, dim=0)), ("roll", dict(shift=shift, dim=1)),
                                   ("slice", dict(dim=0, start=0, stop=SC)), ("slice", dict(dim=1, start=0, stop=SC))])
    y = run1(text, [x])
    assert y.shape == (SC, SC, C)
    for i, j in itertools.product(range(SC), range(SC)):
        np.testing.assert_array_equal(y[i, j], x[(S + i - shift) % S, (S + j - shift) % S])


def test_roll_identities_and_slice_offsets():
    x = f32(np.arange(24).reshape(2, 3, 4))
    np.testing.assert_array_equal(run1(_view_graph((2, 3, 4), [("roll", dict(shift=0, dim=1))]), [x]), x)
    np.testing.assert_array_equal(run1(_view_graph((2, 3, 4), [("roll", dict(shift=3, dim=1))]), [x]), x)
    np.testing.assert_array_equal(run1(_view_graph((2, 3, 4), [("roll", dict(shift=1, dim=2)), ("roll", dict(shift=-1, dim=2))]), [x]), x)
    y = run1(_view_graph((2, 3, 4), [("roll", dict(shift=1, dim=-1))]), [x])
    assert y[0, 0].tolist() == [3, 0, 1, 2]                      # elements move towards higher indices
    z = run1(_view_graph((2, 3, 4), [("slice", dict(dim=2, start=1, stop=3)), ("slice", dict(dim=1, start=2, stop=3))]), [x])
    assert z.shape == (2, 1, 2) and z[1, 0].tolist() == [21, 22]
    # a roll after a slice wraps inside the cut, not inside the source
    w = run1(_view_graph((2, 3, 4), [("slice", dict(dim=2, start=0, stop=3)), ("roll", dict(shift=1, dim=2))]), [x])
    assert w[0, 0].tolist() == [2, 0, 1]


def test_case_1_subgraph_outputs_sum_and_layernorm():
    w = configs.roll_slice_add_layernorm(S=9, SC=6, C=8, dtype="f32")
    add, ln = dag.run(w.text, w.inputs)
    x, r = w.inputs[0].astype(np.float64), w.inputs[1].astype(np.float64)
    want = r + np.roll(x, (3, 3), axis=(0, 1))[:6, :6]
    np.testing.assert_array_equal(add, want)
    v = want.var(axis=-1)
    g, b = w.inputs[2].astype(np.float64), w.inputs[3].astype(np.float64)
    np.testing.assert_allclose(((ln - b) / g).var(axis=-1), v / (v + 1e-5), rtol=1e-10)
    assert np.abs(((ln - b) / g).mean(axis=-1)).max() < 1e-12


# ------------------------------------------------ reductions over the second-to-last dim
def test_column_reductions_match_numpy_and_closed_forms():
    x = f32(np.random.default_rng(5).normal(size=(3, 6, 5)))
    xd = x.astype(np.float64)
    g = Builder()
    i = g.input("f32", x.shape)
    g.output(g.op("sum", [i], "f32", dim=-2, keepdim=0))
    g.output(g.op("mean", [i], "f32", dim=-2))
    g.output(g.op("max", [i], "f32", dim=-2, keepdim=0))
    g.output(g.op("var", [i], "f32", dim=-2, keepdim=0))
    s, m, mx, v = dag.run(g.text(), [x])
    assert s.shape == (3, 5) and m.shape == (3, 1, 5)
    np.testing.assert_allclose(s, xd.sum(axis=1), rtol=1e-14)
    np.testing.assert_allclose(m[:, 0], xd.mean(axis=1), rtol=1e-14, atol=1e-16)
    np.testing.assert_array_equal(mx, xd.max(axis=1))
    np.testing.assert_allclose(v, xd.var(axis=1), rtol=1e-13)
    ones = np.ones((2, 7, 4), np.float32)
    g = Builder()
    i = g.input("f32", ones.shape)
    g.output(g.op("sum", [i], "f32", dim=-2, keepdim=0))
    np.testing.assert_array_equal(dag.run(g.text(), [ones])[0], 7.0)      # counts the 7, not the 4


def test_maximum_minimum_and_nan():
    g = Builder()
    a = g.input("f32", (4,))
    c = g.const(1e-9, "f32")
    g.output(g.op("maximum", [a, c], "f32"))
    g.output(g.op("minimum", [a, c], "f32"))
    hi, lo = dag.run(g.text(), [f32([0.0, 2.0, -1.0, np.nan])])
    assert hi[:3].tolist() == [1e-9, 2.0, 1e-9] and np.isnan(hi[3])
    assert lo[:3].tolist() == [0.0, 1e-9, -1.0] and np.isnan(lo[3])


def test_masked_mean_pooling_is_the_mean_over_unmasked_tokens():
    w = configs.masked_mean_pooling(B=4, S=9, D=6)
    out = dag.run(w.text, w.inputs)[0]
    h = dag.upconvert(w.inputs[1], "bf16")
    assert out.shape == (4, 6)
    for b, n in enumerate(w.meta["lens"]):
        if n == 0:
            np.testing.assert_array_equal(out[b], 0.0)           # 0 / max(0, 1e-9)
        else:
            np.testing.assert_allclose(out[b], h[b, :n].mean(axis=0), rtol=1e-14, atol=1e-16)
    assert w.meta["lens"][0] == 0 and max(w.meta["lens"]) > 1


# ---- IEEE binary16 storage (fp16 task instances) ----

def test_fp16_widening_matches_hand_decoded_patterns_and_every_pattern_of_the_library_type():
    u = np.array([0x3C00, 0x3C01, 0x7BFF, 0x0001, 0x03FF, 0x0400, 0xC000, 0x7C00, 0xFC00, 0x8000, 0x3555], np.uint16)
    got = dag.upconvert(u, "f16")
    want = [1.0, 1.0 + 2.0 ** -10, 65504.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, -2.0, np.inf, -np.inf, -0.0,
            (1024 + 0x155) * 2.0 ** -12]
    np.testing.assert_array_equal(got, want)
    assert np.signbit(got[9]) and np.isnan(dag.upconvert(np.array([0x7E00, 0xFFFF], np.uint16), "f16")).all()
    every = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    lib = every.view(np.float16).astype(np.float64)            # NumPy's own binary16 decoder
    mine = dag.upconvert(every, "f16")
    np.testing.assert_array_equal(np.isnan(mine), np.isnan(lib))
    ok = ~np.isnan(lib)
    np.testing.assert_array_equal(mine[ok], lib[ok])
    np.testing.assert_array_equal(np.signbit(mine[ok]), np.signbit(lib[ok]))


def test_fp16_storage_rounding_is_round_to_nearest_even_in_one_step():
    r = rng.round_to_f16_bits
    x = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -40, 65519.999, 65520.0, 1e6, -1e6,
                  2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -30), 3 * 2.0 ** -25, 2.0 ** -14 - 2.0 ** -25, -0.0, 0.0, np.inf, -np.inf])
    want = [0x3C00, 0x3C02, 0x3C01, 0x7BFF, 0x7C00, 0x7C00, 0xFC00,
            0x0000, 0x0001, 0x0002, 0x0400, 0x8000, 0x0000, 0x7C00, 0xFC00]
    assert r(x).tolist() == want                                # ties to even, overflow to inf, gradual underflow
    assert r(np.array([np.nan]))[0] & 0x7C00 == 0x7C00 and r(np.array([np.nan]))[0] & 0x03FF != 0
    # every finite binary16 value survives a round trip
    every = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = dag.upconvert(every, "f16")
    fin = np.isfinite(vals)
    np.testing.assert_array_equal(r(vals[fin]), every[fin])
    # a double-rounding trap: 1 + 2^-11 + 2^-30 must round up although fp32 would first drop the 2^-30
    assert r(np.array([1.0 + 2.0 ** -11 + 2.0 ** -30]))[0] == 0x3C01
    # agreement with the library's conversion on a few thousand doubles across the range, and monotonicity
    z = rng.normal(11, 0, 4096) * np.exp(rng.normal(11, 1, 4096) * 4.0)
    with np.errstate(over="ignore"):
        np.testing.assert_array_equal(r(z), z.astype(np.float16).view(np.uint16))
    zs = np.sort(np.abs(z))
    zs = zs[zs < 65000.0]
    assert np.all(np.diff(dag.upconvert(r(zs), "f16")) >= 0)


def test_fp16_graphs_are_evaluated_on_the_widened_bits():
    w = configs.cfg3_bias_gelu_gate(rows=3, cols=8, dtype="f16")
    a, bias, b = [dag.upconvert(t, "f16") for t in w.inputs]
    u = a + bias
    want = 0.5 * u * (1 + np.tanh(np.sqrt(2 / np.pi) * (u + 0.044715 * u ** 3))) * b
    np.testing.assert_allclose(dag.run(w.text, w.inputs)[0], want, rtol=1e-14, atol=1e-300)
    m = configs.causal_mask_bits(4, "f16")
    assert np.isneginf(dag.upconvert(m, "f16")[0, 1]) and dag.upconvert(m, "f16")[1, 1] == 0.0
    s = dag.run(configs.cfg2_masked_softmax(heads=1, seq=4, dtype="f16").text, configs.cfg2_masked_softmax(heads=1, seq=4, dtype="f16").inputs)[0]
    np.testing.assert_allclose(s.sum(axis=-1), 1.0, rtol=1e-14)
    assert s[0, 0, 0] == 1.0 and s[0, 0, 1] == 0.0
