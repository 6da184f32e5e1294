"""GPU parity over task instances: one operator sequence at ten shapes (and three dtypes).

The planner's grouping is the rewrite; it has to hold for every member of the instance (the
paper's multi-graph requirement, Sec. 3.1), while the tiling is chosen per member.
"""
import numpy as np
import pytest
import torch

import paper_2605_29357_amd as pf
from tests.harness import Runner, check_against_oracle, to_device
from tests.device import alloc_outputs
from workloads import configs, sweeps

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("family", sweeps.FAMILIES)
def test_every_member_of_the_instance_is_one_kernel_and_matches_the_oracle(family):
    base = pf.Graph(sweeps.member(family, 0).text)
    partitions, tilings = set(), set()
    for k in range(10):
        w = sweeps.member(family, k)
        print(family, k, w.name, flush=True)
        # the member is the base graph at other shapes: the library re-infers every shape itself
        assert base.variant(w.input_shapes).text() == pf.Graph(w.text).text()
        r = Runner(w)
        assert len(r.exe.groups()) == 1                 # one fused group (a column reduction over few tiles runs as
        assert r.info["n_kernels"] <= (2 if family == "masked_mean_pooling" else 1)   # partial + combine kernels)
        gi = r.exe.group_info(0)
        partitions.add(tuple(gi["nodes"]))
        tilings.add((gi["template"], gi["lanes_per_row"], gi["block_threads"], r.exe.source(0).count("pf_ld<")))
        outs = r.run()
        torch.cuda.synchronize()
        check_against_oracle(w, outs, what=w.name)
        del r, outs
    assert len(partitions) == 1                     # the same rewrite for every member
    if family != "bias_gelu_gate":
        assert len(tilings) >= 3, tilings           # but not the same tiling
    last = {sweeps.bucket(s[-1]) for s in sweeps.SHAPES[family]}
    assert {1, 2} <= last


@pytest.mark.parametrize("family,dtypes", [("bias_gelu_gate", ["bf16", "f16", "f32"]), ("masked_softmax", ["bf16", "f16", "f32"]),
                                           ("rmsnorm_rope", ["bf16", "f16"])])
def test_dtype_variants_of_an_instance(family, dtypes):
    base = pf.Graph(sweeps.member(family, 3, dtypes[0]).text)
    for dt in dtypes[1:]:
        for k in (1, 3, 6):
            w = sweeps.member(family, k, dt)
            assert base.variant(w.input_shapes, dtypes[0], dt).text() == pf.Graph(w.text).text()
            r = Runner(w)
            assert r.info["n_kernels"] == 1
            outs = r.run()
            torch.cuda.synchronize()
            check_against_oracle(w, outs, what=w.name)


@pytest.mark.parametrize("name,make,outers", [
    ("flat", lambda r: configs.cfg3_bias_gelu_gate(rows=r, cols=264), (5, 37, 300)),
    ("flat rows of 133, whole vectors", lambda r: configs.cfg3_bias_gelu_gate(rows=r, cols=133, dtype="f32"), (4, 8, 52)),
    ("flat rows of 133, ragged end", lambda r: configs.cfg3_bias_gelu_gate(rows=r, cols=133, dtype="f32"), (5, 7, 49)),
    ("layernorm rows", lambda r: configs.cfg1_add_layernorm(rows=r, cols=768), (7, 64, 200)),
    ("softmax batch", lambda r: configs.cfg2_masked_softmax(heads=r, seq=133), (2, 3, 5)),
    ("rmsnorm + rope batch", lambda r: configs.cfg4_rmsnorm_rope(r, 64, 4, 128), (2, 3, 5)),
    ("layernorm rows streamed", lambda r: configs.cfg1_add_layernorm(rows=r, cols=70001), (2, 3)),
])
def test_members_that_share_one_code_object_match_the_oracle(name, make, outers):
    """Kernels take the outermost extent as an argument: members of an instance that differ only
    there run the same code object (same kernel name = same source hash), each at its own extent."""
    names = set()
    for r in outers:
        w = make(r)
        run = Runner(w)
        assert run.info["n_kernels"] == 1
        names.add(run.exe.kernel_name(0))
        outs = run.run()
        torch.cuda.synchronize()
        check_against_oracle(w, outs, what="%s, outer extent %d" % (name, r))
    assert len(names) == 1, names


@pytest.mark.parametrize("name,make,compiled,others", [
    ("flat", lambda r: configs.cfg3_bias_gelu_gate(rows=r, cols=264), 300, (1, 37, 299)),
    ("layernorm rows", lambda r: configs.cfg1_add_layernorm(rows=r, cols=768), 200, (1, 7, 64)),
    ("layernorm, several rows in flight", lambda r: configs.cfg1_add_layernorm(rows=r, cols=96), 1 << 16, (4, 1000, 65532)),
    ("softmax batch", lambda r: configs.cfg2_masked_softmax(heads=r, seq=133), 5, (2, 3)),
    ("rmsnorm + rope batch", lambda r: configs.cfg4_rmsnorm_rope(r, 64, 4, 128), 5, (2, 4)),
    ("layernorm rows streamed", lambda r: configs.cfg1_add_layernorm(rows=r, cols=70001), 3, (2,)),
])
def test_one_compiled_kernel_runs_smaller_outer_extents(name, make, compiled, others):
    """pf_execute_outer: the kernel compiled for the largest member runs the smaller ones as they come
    (their inputs are other data of the smaller shape), and still runs its own extent afterwards."""
    big = Runner(make(compiled))
    assert big.info["n_kernels"] == 1
    for r in others + (compiled,):
        w = make(r)
        d_in = [to_device(a, dt) for a, dt in zip(w.inputs, w.input_dtypes)]
        outs = alloc_outputs(w)
        big.exe.execute_outer(r, [t.data_ptr() for t in d_in], [t.data_ptr() for t in outs], torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        check_against_oracle(w, outs, what="%s: compiled for %d, run at %d" % (name, compiled, r))
