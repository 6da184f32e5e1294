"""GPU parity of the four named fused subgraphs against the fp64 oracle.

Tolerances (stated by the benchmark spec): |gpu - oracle| <= atol + rtol*|oracle| with
rtol 1e-5 (fp32 outputs) or 2e-2 (bf16 outputs) and atol 1e-5.  Reduced and
full sizes alike are compared element by element; at the full sizes the oracle
evaluates the DAG on blocks of whole rows (every row of these subgraphs is
independent of the others, so a block is a smaller instance of the same DAG).
"""
import numpy as np
import pytest
import torch

from tests.harness import Runner, alloc_outputs, check_against_oracle, check_all_guards, to_host_bits
from oracle import dag as oracle_dag
from workloads import configs
from workloads.irtext import Builder

pytestmark = pytest.mark.gpu


def _run_and_check(w, fuse=True, **kw):
    r = Runner(w, fuse=fuse, **kw)
    outs = r.run()
    torch.cuda.synchronize()
    worst = check_against_oracle(w, outs, what=w.name + (" fused" if fuse else " unfused"))
    return r, worst


@pytest.mark.parametrize("rows,cols", [(64, 768), (3, 768), (7, 96), (5, 100), (2, 4096), (3, 133), (1, 4), (300, 20)])
@pytest.mark.parametrize("use_var_op", [False, True])
def test_cfg1_add_layernorm(rows, cols, use_var_op):
    print("case cfg1", rows, cols, use_var_op, flush=True)
    w = configs.cfg1_add_layernorm(rows=rows, cols=cols, use_var_op=use_var_op)
    r, _ = _run_and_check(w)
    assert r.info["n_kernels"] == 1
    assert r.exe.group_info(0)["template"] == "row_resident"


@pytest.mark.parametrize("heads,seq", [(2, 512), (1, 64), (3, 40), (1, 1024)])
def test_cfg2_masked_softmax(heads, seq):
    print("case cfg2", heads, seq, flush=True)
    w = configs.cfg2_masked_softmax(heads=heads, seq=seq)
    r, _ = _run_and_check(w)
    assert r.info["n_kernels"] == 1
    out = r.run()[0]
    torch.cuda.synchronize()
    got = oracle_dag.upconvert(to_host_bits(out, "bf16"), "bf16")
    iu = np.triu_indices(seq, k=1)
    assert (got[:, iu[0], iu[1]] == 0).all()          # masked entries exactly zero


def test_cfg2_fully_masked_rows_give_nan_like_the_definition():
    w = configs.cfg2_masked_softmax(heads=1, seq=64)
    w.inputs[1][5, :] = 0xFF80
    _run_and_check(w)


@pytest.mark.parametrize("rows,cols", [(16, 11008), (5, 8), (3, 1000), (7, 133), (1, 1)])
def test_cfg3_bias_gelu_gate(rows, cols):
    print("case cfg3", rows, cols, flush=True)
    w = configs.cfg3_bias_gelu_gate(rows=rows, cols=cols)
    r, _ = _run_and_check(w)
    assert r.info["n_kernels"] == 1
    assert r.exe.group_info(0)["template"] == "ew_flat"


@pytest.mark.parametrize("batch,positions,heads,dim", [(1, 16, 4, 128), (2, 33, 3, 64), (1, 5, 1, 6), (2, 8, 32, 128)])
def test_cfg4_rmsnorm_rope(batch, positions, heads, dim):
    print("case cfg4", batch, positions, heads, dim, flush=True)
    w = configs.cfg4_rmsnorm_rope(batch=batch, positions=positions, heads=heads, dim=dim)
    r, _ = _run_and_check(w)
    assert r.info["n_kernels"] == 1


def test_unfused_execution_matches_and_counts_one_kernel_per_node():
    w = configs.cfg1_add_layernorm(rows=9, cols=768)
    r, _ = _run_and_check(w, fuse=False, intermediates_f32=True)
    assert r.info["n_kernels"] == 10
    w = configs.cfg3_bias_gelu_gate(rows=9, cols=1000)
    r, _ = _run_and_check(w, fuse=False, intermediates_f32=True)
    assert r.info["n_kernels"] == 3
    w = configs.cfg2_masked_softmax(heads=1, seq=128)
    r, _ = _run_and_check(w, fuse=False, intermediates_f32=True)
    assert r.info["n_kernels"] == 7
    w = configs.cfg4_rmsnorm_rope(batch=1, positions=9, heads=2, dim=128)
    _run_and_check(w, fuse=False, intermediates_f32=True)


def test_bf16_store_rounds_to_nearest_even_bit_exactly():
    # x + 0 with fp32 input and bf16 output is a pure rounding step
    vals = np.array([1.0, 1.00390625, 1.01171875, 1.005, -2.5, 3.0e38, 1e-40, 0.0, -0.0, np.inf, -np.inf,
                     3.3895313892515355e38], dtype=np.float32)
    rng = np.random.default_rng(0)
    vals = np.concatenate([vals, rng.normal(size=4084).astype(np.float32),
                           rng.integers(0, 2 ** 32, size=4096, dtype=np.uint64).astype(np.uint32).view(np.float32)])
    vals = vals[~np.isnan(vals)][:8000]
    g = Builder()
    i = g.input("f32", (vals.size,))
    g.output(g.op("add", [i, g.const(0.0, "f32")], "bf16"))
    w = configs.Workload("round", g.text(), [vals], ["f32"], [(vals.size,)], ["bf16"], [(vals.size,)]).finish()
    r = Runner(w)
    out = r.run()[0]
    torch.cuda.synchronize()
    from workloads import rng as wrng
    want = wrng.round_to_bf16_bits((vals.astype(np.float64) + 0.0))
    got = to_host_bits(out, "bf16")
    # -0.0 + 0.0 = +0.0 in round-to-nearest
    np.testing.assert_array_equal(got, want)


# ----------------------------------------------------------------- full sizes
def _compare_block(got_bits, ref, dt, what):
    """Every element of one block of rows: |gpu - oracle| <= atol + rtol |oracle|, NaN patterns equal."""
    got = oracle_dag.upconvert(got_bits, dt).reshape(ref.shape)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), what
    err = np.abs(got - ref)
    bound = configs.ATOL[dt] + configs.RTOL[dt] * np.abs(ref)
    bad = ~((got == ref) | (err <= bound))
    assert not bad.any(), "%s: %d elements out of tolerance, worst %g x the bound" % (what, int(bad.sum()), float((err / bound).max()))


def test_cfg3_full_size_every_element():
    """All 8192 x 11008 outputs against the oracle (which evaluates the DAG on blocks of 1024 whole rows: the
    rows of this subgraph are independent, and its fp64 intermediates of the full tensor would take 5 GB)."""
    w = configs.cfg3_bias_gelu_gate()
    r = Runner(w)
    out = r.run()[0]
    torch.cuda.synchronize()
    check_all_guards()
    got = to_host_bits(out, "bf16")
    assert not torch.isnan(out).any()                  # nothing left unwritten (outputs start as NaN)
    step = 1024
    s = configs.cfg3_bias_gelu_gate(rows=step)          # the same DAG on one block of rows
    for r0 in range(0, 8192, step):
        print("cfg3 rows", r0, flush=True)
        s.inputs = [w.inputs[0][r0:r0 + step], w.inputs[1], w.inputs[2][r0:r0 + step]]
        ref = oracle_dag.run(s.text, s.inputs)[0]
        _compare_block(got[r0:r0 + step], ref, "bf16", "cfg3 rows %d.." % r0)


def test_cfg4_full_size_every_element():
    """All 4 x 2048 x 32 x 128 outputs against the oracle, one block of 256 positions of one batch at a time
    (a block uses rows p .. p+255 of the cos / sin tables)."""
    w = configs.cfg4_rmsnorm_rope()
    r = Runner(w)
    out = r.run()[0]
    torch.cuda.synchronize()
    check_all_guards()
    assert not torch.isnan(out).any()
    got = to_host_bits(out, "bf16")
    x = w.inputs[0]
    step = 256
    s = configs.cfg4_rmsnorm_rope(batch=1, positions=step, heads=32, dim=128)     # the same DAG on one block
    for b in range(4):
        for p0 in range(0, 2048, step):
            print("cfg4 batch", b, "positions", p0, flush=True)
            s.inputs = [x[b:b + 1, p0:p0 + step], w.inputs[1], w.inputs[2][p0:p0 + step], w.inputs[3][p0:p0 + step]]
            ref = oracle_dag.run(s.text, s.inputs)[0]
            _compare_block(got[b:b + 1, p0:p0 + step], ref, "bf16", "cfg4 batch %d positions %d.." % (b, p0))


def test_cfg2_full_size():
    w = configs.cfg2_masked_softmax()
    _run_and_check(w)


def test_cfg1_full_size_is_one_kernel_and_repeatable():
    w = configs.cfg1_add_layernorm()
    r, _ = _run_and_check(w)
    a = r.run()[0]
    b = r.run()[0]
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ------------------------------------------------------------- rows too long to stay on chip
def _softmax_workload(rows, cols, dtype, seed=31):
    from workloads import rng as wrng
    g = Builder()
    x = g.input(dtype, (rows, cols))
    m = g.op("max", [x], dtype)
    e = g.op("exp", [g.op("sub", [x, m], dtype)], dtype)
    s = g.op("sum", [e], dtype)
    g.output(g.op("div", [e, s], dtype))
    g.output(s)
    xs = wrng.normal_stored(seed, 0, rows * cols, dtype).reshape(rows, cols)
    return configs.Workload("softmax_%s_%dx%d" % (dtype, rows, cols), g.text(), [xs], [dtype], [(rows, cols)],
                            [dtype, dtype], [(rows, cols), (rows, 1)]).finish()


@pytest.mark.parametrize("rows,cols,dtype", [(3, 70000, "f32"), (2, 100003, "bf16"), (5, 65540, "f32"), (2, 262144, "bf16")])
def test_long_rows_use_the_streaming_row_template(rows, cols, dtype):
    w = _softmax_workload(rows, cols, dtype)
    r, _ = _run_and_check(w)
    assert [gi["template"] for gi in r.exe.groups()] == ["row_loop"]


@pytest.mark.parametrize("use_var_op", [False, True])
def test_long_row_layernorm(use_var_op):
    w = configs.cfg1_add_layernorm(rows=3, cols=70000, use_var_op=use_var_op)
    r, _ = _run_and_check(w)
    assert r.exe.group_info(0)["template"] == "row_loop"


def test_long_row_max_propagates_nan():
    w = _softmax_workload(2, 70000, "f32")
    w.inputs[0][1, 12345] = np.nan
    _run_and_check(w)


def test_a_subgraph_compiled_on_this_machine_runs(tmp_path, monkeypatch):
    """With an empty code-object cache the kernel is specialised and compiled here, then loaded and run."""
    import paper_2605_29357_amd as pf
    monkeypatch.setenv("PF_CACHE_DIR", str(tmp_path))
    w = configs.cfg1_add_layernorm(rows=11, cols=212)          # a shape nothing else uses: not in this process's cache
    before = pf.jit_stats()
    r, _ = _run_and_check(w)
    after = pf.jit_stats()
    assert after["compiled"] == before["compiled"] + 1 and after["disk_hits"] == before["disk_hits"]
    assert len(list(tmp_path.glob("*.pfk"))) == 1
