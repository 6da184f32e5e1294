"""GPU parity for roll / slice folded into the loads of the consuming kernel.

The paper's Case 1 (roll by 3 along two dims, prefix slice, residual add,
LayerNorm, two outputs) must come out as ONE kernel; pure data movement must
be bit-exact.
"""
import numpy as np
import pytest
import torch

from tests.harness import Runner, check_against_oracle, oracle_outputs, to_host_bits
from workloads import configs, rng
from workloads.irtext import Builder

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S,SC,C", [(133, 128, 96), (70, 64, 192), (35, 32, 384), (9, 6, 8), (11, 7, 10)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_case_1_roll_slice_add_layernorm_is_one_kernel(S, SC, C, dtype):
    w = configs.roll_slice_add_layernorm(S=S, SC=SC, C=C, dtype=dtype)
    r = Runner(w)
    assert r.info["n_kernels"] == 1 and r.info["workspace_bytes"] == 0
    assert r.exe.group_info(0)["template"] == "row_resident"
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, what=w.name)
    u = Runner(w, fuse=False, intermediates_f32=True)
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, what=w.name + " unfused")


def _movement_case(shape, steps, tail=None, dtype="f32", seed=77):
    """A chain of views, optionally followed by ops; returns the workload."""
    g = Builder()
    t = g.input(dtype, shape)
    for op, attrs in steps:
        t = g.op(op, [t], dtype, **attrs)
    if tail:
        t = tail(g, t)
    outs = t if isinstance(t, list) else [t]
    for o in outs:
        g.output(o)
    x = rng.normal_stored(seed, 0, int(np.prod(shape)), dtype).reshape(shape)
    w = configs.Workload("views", g.text(), [x], [dtype], [tuple(shape)], [dtype] * len(outs), [()] * len(outs))
    refs = oracle_outputs(w)
    w.output_shapes = [r.shape for r in refs]
    return w.finish(), refs


CASES = [
    ((6, 10, 16), [("roll", dict(shift=2, dim=0))]),
    ((6, 10, 16), [("roll", dict(shift=-3, dim=1)), ("slice", dict(dim=1, start=2, stop=9))]),
    ((6, 10, 16), [("roll", dict(shift=5, dim=2))]),                                  # along the contiguous dim
    ((6, 10, 16), [("slice", dict(dim=2, start=3, stop=11)), ("roll", dict(shift=1, dim=2))]),
    ((6, 10, 16), [("slice", dict(dim=0, start=4, stop=5)), ("roll", dict(shift=7, dim=1))]),   # a dim collapses to 1
    ((40, 133), [("roll", dict(shift=3, dim=0)), ("roll", dict(shift=131, dim=1)), ("slice", dict(dim=0, start=1, stop=33))]),
    ((3, 5, 7, 9), [("roll", dict(shift=1, dim=0)), ("roll", dict(shift=2, dim=1)), ("roll", dict(shift=3, dim=2)),
                    ("slice", dict(dim=3, start=0, stop=8))]),
    ((300, 2048), [("slice", dict(dim=0, start=10, stop=290)), ("roll", dict(shift=100, dim=0))]),
]


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_view_chains_move_data_bit_exactly(case, dtype):
    shape, steps = CASES[case]
    w, refs = _movement_case(shape, steps, dtype=dtype)
    for fuse in (True, False):
        r = Runner(w, fuse=fuse)
        assert r.info["n_kernels"] == 1            # the chain folds into one copy kernel either way
        out = r.run()[0]
        torch.cuda.synchronize()
        from oracle import dag as oracle_dag
        got = oracle_dag.upconvert(to_host_bits(out, dtype), dtype)
        np.testing.assert_array_equal(got, refs[0])


def test_views_feed_reductions_transposes_and_long_rows():
    # view -> softmax-like row kernel with a second output
    def tail(g, t):
        m = g.op("max", [t], "f32")
        e = g.op("exp", [g.op("sub", [t, m], "f32")], "f32")
        return [g.op("div", [e, g.op("sum", [e], "f32")], "f32"), m]
    w, refs = _movement_case((50, 300), [("roll", dict(shift=7, dim=1)), ("slice", dict(dim=0, start=5, stop=45))], tail)
    r = Runner(w)
    assert r.info["n_kernels"] == 1
    check_against_oracle(w, r.run(), refs=refs)
    # view -> transpose (the window is materialised first) -> tanh
    w, refs = _movement_case((64, 96), [("roll", dict(shift=3, dim=0))],
                             lambda g, t: g.op("tanh", [g.op("transpose", [t], "f32")], "f32"))
    r = Runner(w)
    check_against_oracle(w, r.run(), refs=refs)
    # transpose -> view of the transposed tensor -> add
    def tail2(g, t):
        v = g.op("roll", [g.op("transpose", [t], "f32")], "f32", shift=2, dim=1)
        return g.op("add", [v, g.const(1.0, "f32")], "f32")
    w, refs = _movement_case((48, 80), [], tail2)
    check_against_oracle(w, Runner(w).run(), refs=refs)
    # view of a computed value: the producer is stored, the consumer gathers
    def tail3(g, t):
        e = g.op("exp", [t], "f32")
        v = g.op("slice", [g.op("roll", [e], "f32", shift=1, dim=0)], "f32", dim=1, start=8, stop=40)
        return [g.op("mul", [v, v], "f32"), e]
    w, refs = _movement_case((33, 64), [], tail3)
    r = Runner(w)
    assert r.info["n_kernels"] == 2
    check_against_oracle(w, r.run(), refs=refs)
    # a rolled row that is too long to stay on chip
    def tail4(g, t):
        return g.op("sub", [t, g.op("mean", [t], "f32")], "f32")
    w, refs = _movement_case((2, 70000), [("roll", dict(shift=12345, dim=1))], tail4)
    r = Runner(w)
    assert r.exe.group_info(0)["template"] == "row_loop"
    check_against_oracle(w, r.run(), refs=refs)
    torch.cuda.synchronize()
