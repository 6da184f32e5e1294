"""GPU parity for transposes of computed values.

The planner pushes a transpose of an elementwise value down to the operands (the consumer's
kernel recomputes the value in its own orientation; operands with a last or second-to-last
extent of 1 change orientation without moving data).  The oracle executes the graph as written,
transposes included, so these cases check the rewrite against the definition.
"""
import numpy as np
import pytest
import torch

from tests.harness import Runner, check_against_oracle, oracle_outputs
from workloads import configs, rng
from workloads.irtext import Builder

pytestmark = pytest.mark.gpu


def _workload(name, build, shapes, dtype, positive=()):
    g = Builder()
    ins = [g.input(dtype, s) for s in shapes]
    outs = build(g, ins)
    for o in outs:
        g.output(o)
    data = []
    for k, s in enumerate(shapes):
        x = rng.normal(90 + k, 0, int(np.prod(s))).reshape(s)
        if k in positive:
            x = np.abs(x) + 0.5
        data.append(rng.store(x, dtype))
    w = configs.Workload(name, g.text(), data, [dtype] * len(shapes), [tuple(s) for s in shapes], [dtype] * len(outs),
                         [()] * len(outs))
    refs = oracle_outputs(w)
    w.output_shapes = [r.shape for r in refs]
    return w.finish(), refs


def _softmax_then_transpose(g, ins):
    x, wgt = ins
    m = g.op("max", [x], g_dt(g))
    e = g.op("exp", [g.op("sub", [x, m], g_dt(g))], g_dt(g))
    p = g.op("div", [e, g.op("sum", [e], g_dt(g))], g_dt(g))
    return [g.op("mul", [g.op("transpose", [p], g_dt(g)), wgt], g_dt(g))]


def g_dt(g):
    return g.dtype


CASES = [
    # (name, builder, input shapes, indices of inputs kept positive, expected kernels)
    ("unary chain", lambda g, i: [g.op("tanh", [g.op("transpose", [g.op("exp", [i[0]], g.dtype)], g.dtype)], g.dtype)],
     [(70, 133)], (), 1),
    ("weights and per-row scale change orientation for free",
     lambda g, i: [g.op("gelu", [g.op("transpose", [g.op("mul", [g.op("add", [i[0], i[1]], g.dtype), i[2]], g.dtype)], g.dtype)], g.dtype)],
     [(96, 200), (200,), (96, 1)], (), 1),
    ("two full operands", lambda g, i: [g.op("sub", [g.op("transpose", [g.op("div", [i[0], i[1]], g.dtype)], g.dtype), i[2]], g.dtype)],
     [(133, 64), (133, 64), (64, 133)], (1,), 1),
    ("needed in both orientations",
     lambda g, i: (lambda e: [e, g.op("tanh", [g.op("transpose", [e], g.dtype)], g.dtype)])(g.op("exp", [i[0]], g.dtype)),
     [(3, 50, 72)], (), 1),          # one tile kernel computes it in the transposed orientation and stores it both ways
    ("results of both orientations from the same tensor leave one tile kernel",
     lambda g, i: (lambda e: [g.op("transpose", [g.op("add", [e, g.const(0.587, g.dtype)], g.dtype)], g.dtype), g.op("exp", [i[0]], g.dtype),
                              g.op("transpose", [g.op("tanh", [e], g.dtype)], g.dtype)])(g.op("exp", [i[0]], g.dtype)),
     [(133, 70)], (), 1),
    ("a result of the other orientation that needs one more tensor is taken over as well",
     lambda g, i: [g.op("div", [g.op("sub", [i[0], i[1]], g.dtype), i[1]], g.dtype),
                   g.op("tanh", [g.op("transpose", [g.op("gelu", [g.op("rsqrt", [i[1]], g.dtype)], g.dtype, approx="tanh")], g.dtype)], g.dtype)],
     [(5, 61, 96), (5, 61, 96)], (1,), 1),
    ("a transpose only the caller reads is written by the kernel that computes its operand",
     lambda g, i: (lambda v: [g.op("transpose", [g.op("tanh", [v], g.dtype)], g.dtype), g.op("add", [v, i[2]], g.dtype)])(
         g.op("sub", [i[0], i[1]], g.dtype)),
     [(3, 96, 259), (96, 1), (3, 96, 259)], (), 1),
    ("batched, scalar constant inside the cone",
     lambda g, i: [g.op("add", [g.op("transpose", [g.op("mul", [g.op("sigmoid", [i[0]], g.dtype), g.const(1.5, g.dtype)], g.dtype)], g.dtype), i[1]], g.dtype)],
     [(4, 33, 80), (80, 1)], (), 1),
    ("softmax, then transposed and scaled: only the row statistics cross kernels", _softmax_then_transpose, [(64, 96), (96, 1)], (), 2),
    ("transposed twice", lambda g, i: [g.op("exp", [g.op("transpose", [g.op("transpose", [g.op("tanh", [i[0]], g.dtype)], g.dtype)], g.dtype)], g.dtype)],
     [(40, 56)], (), 1),
    ("a reduction behind the recomputed value",
     lambda g, i: (lambda h: [g.op("div", [h, g.op("sum", [h], g.dtype)], g.dtype)])(
         g.op("transpose", [g.op("exp", [g.op("mul", [i[0], g.const(0.1, g.dtype)], g.dtype)], g.dtype)], g.dtype)),
     [(48, 100)], (), 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,build,shapes,positive,kernels", CASES)
def test_transposes_of_computed_values_match_the_oracle(name, build, shapes, positive, kernels, dtype):
    def build_typed(g, ins):
        g.dtype = dtype
        return build(g, ins)
    w, refs = _workload(name, build_typed, shapes, dtype, positive)
    r = Runner(w)
    assert r.info["n_kernels"] == kernels, (name, [gi["template"] for gi in r.exe.groups()])
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, refs=refs, what=name)
    u = Runner(w, fuse=False, intermediates_f32=True)          # op by op: every transpose is a kernel of its own
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, refs=refs, what=name + " unfused")


@pytest.mark.parametrize("dtype,shape", [("bf16", (4096, 4096)), ("bf16", (4100, 4099)), ("f32", (2, 1999, 2050)), ("f16", (3, 1000, 2056))])
def test_large_tiles_store_results_of_both_orientations(dtype, shape):
    """64-wide tiles with a store through the LDS transpose: x * w in x's own orientation and its transpose (plus an
    epilogue) leave one kernel; whole and ragged extents, 16- and 32-bit elements."""
    t_shape = tuple(shape[:-2]) + (shape[-1], shape[-2])

    def build(g, ins):
        g.dtype = dtype
        y = g.op("mul", [ins[0], ins[1]], dtype)                                   # [.., R, C], stays an output in this orientation
        return [y, g.op("add", [g.op("transpose", [y], dtype), ins[2]], dtype)]     # [.., C, R]
    w, refs = _workload("both orientations", build, [shape, (shape[-1],), t_shape], dtype)
    r = Runner(w)
    assert r.info["n_kernels"] == 1 and r.exe.group_info(0)["template"] == "tile"
    assert r.info["planned_bytes"] == w.algorithmic_bytes
    if shape[-1] >= 4096:
        assert "TS = 64" in r.exe.source(0)
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, refs=refs, what="both orientations %s %s" % (dtype, shape))
    u = Runner(w, fuse=False, intermediates_f32=True)
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, refs=refs, what="both orientations unfused")


@pytest.mark.parametrize("dtype,shape", [("bf16", (4096, 4096)), ("f16", (2, 3000, 2056)), ("bf16", (4100, 4099)), ("bf16", (3, 2999, 3001)),
                                         ("f32", (4096, 4096))])
def test_large_transposes_with_an_epilogue(dtype, shape):
    """64-wide tiles (eight-element vectors when every tensor of the group holds 16-bit elements), whole and
    ragged extents; pure data movement must be bit-exact."""
    t_shape = tuple(shape[:-2]) + (shape[-1], shape[-2])

    def build(g, ins):
        g.dtype = dtype
        t = g.op("transpose", [ins[0]], dtype)
        return [t, g.op("mul", [g.op("add", [t, ins[1]], dtype), ins[2]], dtype)]
    w, refs = _workload("large transpose", build, [shape, t_shape, (t_shape[-1],)], dtype)
    r = Runner(w)
    assert r.info["n_kernels"] == 1 and r.exe.group_info(0)["template"] == "tile"
    assert "TS = 64" in r.exe.source(0) and ("VW = 8" in r.exe.source(0)) == (dtype != "f32")
    outs = r.run()
    torch.cuda.synchronize()
    from tests.harness import to_host_bits
    moved = to_host_bits(outs[0], dtype)
    np.testing.assert_array_equal(moved, np.swapaxes(w.inputs[0], -1, -2))      # the bits themselves
    check_against_oracle(w, outs, refs=refs, what="large transpose %s %s" % (dtype, shape))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_side_computations_ride_on_another_kernel(dtype):
    """A chain on a weight vector and one on per-row scalars would each be a one-workgroup kernel; independent of the
    main kernel, they run as extra workgroups of it: one launch, four outputs."""
    R, C = 300, 96

    def build(g, ins):
        g.dtype = dtype
        x, wgt, per_row = ins                                                     # [R,C], [C], [R,1]
        main = g.op("mul", [g.op("sub", [x, g.op("mean", [x], dtype)], dtype), wgt], dtype)
        side_w = g.op("mul", [g.op("sigmoid", [wgt], dtype), g.const(2.0, dtype)], dtype)
        side_sum = g.op("sum", [g.op("exp", [wgt], dtype)], dtype)
        return [main, side_w, side_sum, g.op("tanh", [per_row], dtype)]
    w, refs = _workload("riders", build, [(R, C), (C,), (R, 1)], dtype)
    r = Runner(w)
    assert r.info["n_kernels"] == 1 and "pf_rider1" in r.exe.source(0)
    outs = r.run()
    torch.cuda.synchronize()
    check_against_oracle(w, outs, refs=refs, what="riders " + dtype)
    u = Runner(w, fuse=False, intermediates_f32=True)
    assert u.info["n_kernels"] == 8
    uo = u.run()
    torch.cuda.synchronize()
    check_against_oracle(w, uo, refs=refs, what="riders unfused")
