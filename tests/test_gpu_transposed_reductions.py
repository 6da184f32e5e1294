"""GPU parity for reductions over the last dim of values that only exist transposed.

reduce(f(transpose(a), b), last dim) equals a reduction over the second-to-last dim of f evaluated in a's own
orientation, so the compiler may run it as a column reduction that reads a as it lies in memory and hand the
result ([.., R, 1] and [.., 1, R] have the same linear order) to readers in either orientation.  Each case here
is checked against the fp64 oracle, fused and op by op, and the plan is checked to be the one that avoids moving
the transposed value through memory.
"""
import numpy as np
import pytest

from tests.test_gpu_colreduce import _run_both, _workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("op", ["sum", "mean", "max", "var"])
@pytest.mark.parametrize("keepdim", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(70, 96), (3, 45, 133), (2, 3, 9, 40)])
def test_reduction_of_a_transposed_input(op, keepdim, dtype, shape):
    attrs = dict(keepdim=keepdim)
    if op == "var":
        attrs["correction"] = 1

    def build(g, ins):
        t = g.op("transpose", [ins[0]], dtype)
        return [(g.op(op, [t], dtype, **attrs), dtype)]

    w, refs = _workload("t_%s" % op, build, [shape], [dtype])
    want = list(shape[:-2]) + ([shape[-1], 1] if keepdim else [shape[-1]])
    assert refs[0].shape == tuple(want)
    # one kernel that reads the input once, in its own orientation
    _run_both(w, refs, kernels=1, template=["col_reduce"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("R,C", [(96, 70), (133, 257), (64, 2100)])
def test_statistic_of_a_transposed_cone_feeds_both_orientations(dtype, R, C):
    # a: [C, R] in memory; everything below lives on [R, C].  The mean over the last dim of the transposed cone is
    # read back by a full value in the transposed orientation (tile kernel) and by an epilogue of the reduced shape.
    def build(g, ins):
        a, wgt, col, b = ins                                   # [C,R], [R,1], [C], [R,C]
        t = g.op("transpose", [a], dtype)
        x = g.op("add", [g.op("sub", [t, wgt], dtype), col], dtype)
        m = g.op("mean", [x], dtype)                           # [R,1]
        y = g.op("mul", [x, m], dtype)                         # full, transposed orientation
        z = g.op("sub", [g.op("tanh", [m], dtype), wgt], dtype)   # reduced shape
        o2 = g.op("add", [y, b], dtype)
        return [(o2, dtype), (z, dtype), (m, dtype)]

    w, refs = _workload("t_cone", build, [(C, R), (R, 1), (C,), (R, C)], [dtype] * 4, scale=0.5)
    assert [r.shape for r in refs] == [(R, C), (R, 1), (R, 1)]
    r = _run_both(w, refs)
    if C == 2100:
        # 2100 rows of 64 columns in a's orientation: the column reduction would be split over workgroups, which
        # costs a third launch; on a problem this small the traffic model keeps the transpose in front of a row kernel
        assert r.info["n_kernels"] == 2
        return
    assert [gi["template"] for gi in r.exe.groups()] == ["col_reduce", "tile"]
    # a and b read, o2 written, a read once more for the statistic; nothing full-size crosses kernels
    item = 4 if dtype == "f32" else 2
    assert r.info["planned_bytes"] < w.algorithmic_bytes + 1.5 * R * C * item
    assert r.info["workspace_bytes"] < R * C * item


def test_softmax_over_the_rows_of_a_transposed_input():
    # max and sum both run in the input's orientation when that moves fewer bytes; whichever plan is
    # chosen, the values must match
    def build(g, ins):
        t = g.op("transpose", [ins[0]], "f32")
        mx = g.op("max", [t], "f32")
        e = g.op("exp", [g.op("sub", [t, mx], "f32")], "f32")
        s = g.op("sum", [e], "f32")
        return [(g.op("div", [e, s], "f32"), "f32")]

    w, refs = _workload("t_softmax", build, [(300, 200)], ["f32"])
    np.testing.assert_allclose(refs[0].sum(axis=-1), 1.0, rtol=1e-12)
    _run_both(w, refs)


def test_reduction_result_read_through_a_further_transpose_keeps_the_plain_plan():
    # a reader that is not elementwise (here: a transpose of the statistic) is not taught to take the result
    # as it lies, so the reduction stays a row reduction behind the transpose
    def build(g, ins):
        t = g.op("transpose", [ins[0]], "f32")
        m = g.op("sum", [g.op("exp", [t], "f32")], "f32")          # [R,1]
        mt = g.op("transpose", [m], "f32")                         # [1,R]
        return [(g.op("mul", [ins[1], mt], "f32"), "f32")]

    w, refs = _workload("t_further", build, [(80, 48), (5, 48)], ["f32"] * 2, scale=0.3)
    r = _run_both(w, refs)
    assert "col_reduce" not in [gi["template"] for gi in r.exe.groups()]
