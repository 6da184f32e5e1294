"""GPU parity for reductions over the second-to-last dim and maximum / minimum.

The paper's Case 2 (masked mean pooling: two sums over the sequence dim, a
clamp of the denominator, a division) must come out as ONE kernel whose
output matches the fp64 oracle within the fp32 tolerance.
"""
import numpy as np
import pytest
import torch

from tests.harness import Runner, check_against_oracle, oracle_outputs
from workloads import configs, rng
from workloads.irtext import Builder

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,S,D", [(4, 128, 256), (3, 50, 133), (1, 7, 8), (2, 1, 40), (5, 1000, 24), (2, 300, 1), (16, 33, 1024),
                                   (1, 2048, 512), (2, 4099, 48), (3, 777, 133)])
def test_case_2_masked_mean_pooling_is_one_kernel(B, S, D):
    w = configs.masked_mean_pooling(B=B, S=S, D=D)
    r = Runner(w)
    assert len(r.exe.groups()) == 1 and r.exe.group_info(0)["template"] == "col_reduce"
    # few (batch, column tile) pairs and many tokens: the rows are split over workgroups and a second,
    # small kernel combines the partial sums (they cross the workspace)
    split = r.info["n_kernels"] == 2
    assert r.info["n_kernels"] in (1, 2) and (r.info["workspace_bytes"] > 0) == split
    assert split == ((B, S, D) in [(1, 2048, 512), (2, 4099, 48), (3, 777, 133)])
    if not split:
        assert r.info["planned_bytes"] == w.algorithmic_bytes
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, what=w.name)
    got = outs[0].cpu().numpy().reshape(B, D)
    assert np.all(got[0] == 0.0)                                   # fully masked sequence: 0 / 1e-9
    u = Runner(w, fuse=False, intermediates_f32=True)
    assert u.info["n_groups"] == 5
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, what=w.name + " unfused")


def _workload(name, build, shapes, dtypes, seed=91, scale=1.0):
    g = Builder()
    ins = [g.input(dt, sh) for sh, dt in zip(shapes, dtypes)]
    outs = build(g, ins)
    for o, _ in outs:
        g.output(o)
    data = []
    for k, (sh, dt) in enumerate(zip(shapes, dtypes)):
        x = rng.normal(seed, k, int(np.prod(sh))) * scale
        data.append(rng.store(x, dt).reshape(sh))
    w = configs.Workload(name, g.text(), data, list(dtypes), [tuple(s) for s in shapes], [dt for _, dt in outs], [()] * len(outs))
    refs = oracle_outputs(w)
    w.output_shapes = [r.shape for r in refs]
    return w.finish(), refs


def _run_both(w, refs, kernels=None, template=None):
    r = Runner(w)
    if kernels is not None:
        assert r.info["n_kernels"] == kernels, [gi["template"] for gi in r.exe.groups()]
    if template is not None:
        assert [gi["template"] for gi in r.exe.groups()] == template
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, refs=refs, what=w.name)
    u = Runner(w, fuse=False, intermediates_f32=True)
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, refs=refs, what=w.name + " unfused")
    return r


@pytest.mark.parametrize("op", ["sum", "mean", "max", "var"])
@pytest.mark.parametrize("keepdim", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(3, 70, 96), (37, 20), (2, 3, 9, 130)])
def test_single_column_reductions(op, keepdim, dtype, shape):
    attrs = dict(dim=-2, keepdim=keepdim)
    if op == "var":
        attrs["correction"] = 1

    def build(g, ins):
        return [(g.op(op, [ins[0]], dtype, **attrs), dtype)]

    w, refs = _workload("col_%s" % op, build, [shape], [dtype])
    want = list(shape)
    want[-2:] = [1, shape[-1]] if keepdim else [shape[-1]]
    assert refs[0].shape == tuple(want)
    _run_both(w, refs, kernels=1, template=["col_reduce"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prologue_epilogue_and_operands_in_both_alignments(dtype):
    B, S, D = 4, 45, 72

    # keepdim=1: the epilogue lives on [B,1,D]; per-batch scale [B,1,1], weight [D], bias [B,1,D]
    def build_keep(g, ins):
        x, y, wgt, sc, bias = ins
        t = g.op("mul", [g.op("add", [x, y], dtype), wgt], dtype)          # prologue, broadcast operand along S
        t = g.op("tanh", [t], dtype)
        m = g.op("mean", [t], dtype, dim=-2, keepdim=1)
        mx = g.op("max", [x], dtype, dim=-2, keepdim=1)
        e = g.op("add", [g.op("mul", [g.op("sub", [mx, m], dtype), sc], dtype), bias], dtype)
        e = g.op("minimum", [g.op("mul", [e, g.const(0.5, dtype)], dtype), wgt], dtype)
        return [(e, dtype), (t, dtype), (m, dtype)]                        # epilogue value, full value, a reduction itself

    w, refs = _workload("col_keep", build_keep, [(B, S, D), (B, S, D), (D,), (B, 1, 1), (B, 1, D)], [dtype] * 5)
    assert [r.shape for r in refs] == [(B, 1, D), (B, S, D), (B, 1, D)]
    _run_both(w, refs, kernels=1, template=["col_reduce"])

    # keepdim=0: the epilogue lives on [B,D]; weight [D], bias [B,D], per-batch scale [B,1]
    def build_drop(g, ins):
        x, y, wgt, sc, bias = ins
        t = g.op("sigmoid", [g.op("mul", [x, y], dtype)], dtype)            # y is [1,S,1]: one value per row
        s = g.op("sum", [t], dtype, dim=-2, keepdim=0)
        v = g.op("var", [x], dtype, dim=-2, keepdim=0, correction=0)
        e = g.op("mul", [g.op("add", [g.op("mul", [s, wgt], dtype), bias], dtype), sc], dtype)
        e = g.op("div", [e, g.op("maximum", [v, g.const(0.25, dtype)], dtype)], dtype)
        return [(e, dtype)]

    w, refs = _workload("col_drop", build_drop, [(B, S, D), (1, S, 1), (D,), (B, 1), (B, D)], [dtype] * 5)
    assert refs[0].shape == (B, D)
    _run_both(w, refs, kernels=1, template=["col_reduce"])


def test_full_consumers_of_a_column_reduction_start_a_new_kernel():
    # softmax over the sequence dim: max -> exp(x - max) -> sum -> div; each value of the reduced
    # shape is read back as a broadcast operand by the next kernel
    def build(g, ins):
        x = ins[0]
        mx = g.op("max", [x], "f32", dim=-2, keepdim=1)
        e = g.op("exp", [g.op("sub", [x, mx], "f32")], "f32")
        s = g.op("sum", [e], "f32", dim=-2, keepdim=1)
        return [(g.op("div", [e, s], "f32"), "f32")]

    w, refs = _workload("col_softmax", build, [(3, 41, 100)], ["f32"])
    np.testing.assert_allclose(refs[0].sum(axis=-2), 1.0, rtol=1e-12)
    _run_both(w, refs, kernels=3, template=["col_reduce", "col_reduce", "ew_flat"])

    # keepdim=0 result consumed by a full node: [D] lines up with the last dim
    def build0(g, ins):
        x = ins[0]
        m = g.op("mean", [x], "f32", dim=-2, keepdim=0)
        return [(g.op("sub", [x, m], "f32"), "f32")]

    w, refs = _workload("col_center", build0, [(41, 100)], ["f32"])
    np.testing.assert_allclose(refs[0].mean(axis=0), 0.0, atol=1e-12)
    _run_both(w, refs, kernels=2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_split_rows_cover_sum_mean_max_and_ragged_tails(dtype):
    # 3 x 2 column tiles only, 5003 rows: split; the last row segments are short or empty
    def build(g, ins):
        x, y = ins
        t = g.op("mul", [x, y], dtype)
        s = g.op("sum", [t], dtype, dim=-2, keepdim=1)
        m = g.op("mean", [x], dtype, dim=-2, keepdim=1)
        mx = g.op("max", [t], dtype, dim=-2, keepdim=1)
        e = g.op("add", [g.op("mul", [s, g.const(1e-2, dtype)], dtype), g.op("sub", [mx, m], dtype)], dtype)
        return [(e, dtype), (mx, dtype), (t, dtype)]

    w, refs = _workload("col_split", build, [(3, 5003, 200), (1, 5003, 1)], [dtype] * 2)
    r = Runner(w)
    assert len(r.exe.groups()) == 1 and r.info["n_kernels"] == 2
    _run_both(w, refs)
    # a variance needs the mean of the whole column first: never split
    w, refs = _workload("col_var_long", lambda g, ins: [(g.op("var", [ins[0]], dtype, dim=-2, keepdim=0), dtype)], [(2, 3000, 40)], [dtype])
    assert Runner(w).info["n_kernels"] == 1
    _run_both(w, refs, kernels=1)
    # NaN in one row segment reaches the column maximum
    x = rng.normal(5, 0, 2048 * 64).astype(np.float32).reshape(1, 2048, 64)
    x[0, 1777, 5] = np.nan
    g = Builder()
    a = g.input("f32", x.shape)
    g.output(g.op("max", [a], "f32", dim=-2, keepdim=0))
    w = configs.Workload("col_split_nan", g.text(), [x], ["f32"], [x.shape], ["f32"], [(1, 64)]).finish()
    refs = oracle_outputs(w)
    assert np.isnan(refs[0][0, 5]) and np.isnan(refs[0]).sum() == 1
    assert Runner(w).info["n_kernels"] == 2
    _run_both(w, refs)


def test_nan_propagates_through_column_max_and_maximum_minimum():
    S, D = 19, 48
    x = rng.normal(5, 0, S * D).astype(np.float32).reshape(S, D)
    x[7, 3] = np.nan
    x[0, 11] = np.inf
    x[18, 47] = -np.inf
    y = rng.normal(5, 1, D).astype(np.float32)
    y[5] = np.nan
    g = Builder()
    a = g.input("f32", (S, D))
    b = g.input("f32", (D,))
    mx = g.op("max", [a], "f32", dim=-2, keepdim=0)
    g.output(g.op("maximum", [mx, b], "f32"))
    g.output(g.op("minimum", [a, b], "f32"))
    w = configs.Workload("col_nan", g.text(), [x, y], ["f32", "f32"], [(S, D), (D,)], ["f32", "f32"], [(D,), (S, D)]).finish()
    refs = oracle_outputs(w)
    assert np.isnan(refs[0][3]) and np.isnan(refs[0][5]) and np.isposinf(refs[0][11]) and np.isnan(refs[1][:, 5]).all()
    _run_both(w, refs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_maximum_minimum_in_flat_and_row_kernels(dtype):
    def build(g, ins):
        x, y = ins
        c = g.op("minimum", [g.op("maximum", [x, g.const(-0.5, dtype)], dtype), g.const(0.75, dtype)], dtype)   # clamp
        r = g.op("max", [g.op("maximum", [x, y], dtype)], dtype)                                              # row kernel
        return [(c, dtype), (g.op("minimum", [g.op("sub", [x, r], dtype), y], dtype), dtype)]

    w, refs = _workload("minmax", build, [(33, 130), (130,)], [dtype] * 2)
    assert refs[0].min() == -0.5 and refs[0].max() == 0.75
    _run_both(w, refs)


def test_case_2_at_the_paper_shape_spot_checks_and_timing():
    w = configs.masked_mean_pooling()                              # B=32, S=512, D=1024
    r = Runner(w)
    assert r.info["n_kernels"] == 1
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, what=w.name)
