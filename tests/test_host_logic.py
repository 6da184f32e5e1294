"""Host-only tests of the library: IR, shape inference, text round trip, planner,
kernel specialisation (JIT for gfx950 needs no GPU) and the exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_29357_amd as pf
from oracle import dag as oracle_dag
from workloads import configs, dags
from workloads.irtext import Builder

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pf.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pf_[a-z0-9_]+)\s*\(", hdr))
    assert {"pf_compile", "pf_execute", "pf_score", "pf_graph_parse", "pf_exec_info", "pf_copy_bytes"} <= names
    L = ctypes.CDLL(pf.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), n
    assert pf.version().startswith("pf ")


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(pf.ScoreResult) == 80
    assert ctypes.sizeof(pf.Pair) == 56


def test_text_round_trip_and_shape_inference_agree_with_the_oracle_reader():
    for w in [configs.cfg1_add_layernorm(rows=4, cols=8), configs.cfg2_masked_softmax(heads=2, seq=8),
              configs.cfg3_bias_gelu_gate(rows=4, cols=8), configs.cfg4_rmsnorm_rope(1, 4, 2, 8),
              configs.roll_slice_add_layernorm(S=9, SC=6, C=8), configs.masked_mean_pooling(B=2, S=5, D=8)] + \
             [dags.cfg5(k, max_rows=4) for k in range(0, 256, 17)]:
        g = pf.Graph(w.text)
        t1 = g.text()
        g2 = pf.Graph(t1)
        assert g2.text() == t1                                   # print -> parse -> print is a fixed point
        og = oracle_dag.parse(w.text)
        oracle_dag.run(og, w.inputs)                             # fills the oracle's shapes
        n_nodes, n_in, n_out = g.size()
        assert n_nodes == len(og.nodes) and n_in == len(og.inputs) and n_out == len(og.outputs)
        for i, on in enumerate(og.nodes):
            ni = g.node_info(i)
            assert ni["op"] == on.op and ni["shape"] == tuple(on.shape), (i, ni, on.op, on.shape)
            assert ni["inputs"] == list(on.args)
            assert ni["is_output"] == (i in og.outputs)


def test_node_by_node_construction_equals_parsing():
    g = pf.Graph()
    a = g.input("bf16", (6, 10))
    b = g.input("bf16", (10,))
    c = g.node("add", [a, b], "bf16")
    d = g.node("gelu", [c], "bf16", approx="erf")
    e = g.node("var", [d], "f32", correction=1, keepdim=0)
    k = g.node("const", [], "f32", value=0.5)
    f = g.node("mul", [e, k], "f32")
    g.output(f)
    assert g.node_info(e)["shape"] == (6,)
    assert pf.Graph(g.text()).text() == g.text()
    assert "approx=erf" in g.text() and "correction=1" in g.text()


@pytest.mark.parametrize("text,frag", [
    ("in %0 : f32[4]\n%1 = add(%0) : f32\nout %1\n", "takes 2"),
    ("in %0 : f32[4]\nin %1 : f32[5]\n%2 = add(%0, %1) : f32\nout %2\n", "broadcast"),
    ("in %0 : f32[4]\n%1 = frob(%0) : f32\nout %1\n", "unknown operator"),
    ("in %0 : f64[4]\n%1 = exp(%0) : f32\nout %1\n", "dtype"),
    ("in %0 : f32[4]\n%2 = exp(%0) : f32\nout %2\n", "consecutive"),
    ("in %0 : f32[4]\n%1 = exp(%1) : f32\nout %1\n", "earlier"),
    ("in %0 : f32[4]\n%1 = transpose(%0) : f32\nout %1\n", "rank"),
    ("in %0 : f32[4,3]\n%1 = rot_pairs(%0) : f32\nout %1\n", "even"),
    ("in %0 : f32[4,0]\n", "positive"),
    ("in %0 : f32[2,2,2,2,2]\n", "rank"),
    ("in %0 : f32[4]\n%1 = exp(%0) {keepdim=1} : f32\nout %1\n", "not valid"),
    ("in %0 : f32[4]\n%1 = const() : f32\n", "value"),
    ("in %0 : f32[4]\n%1 = exp(%0) : f32\n", "no outputs"),
    ("in %0 : f32[4]\nout %0\n", "graph input"),
    ("in %0 : f32[4,6]\n%1 = sum(%0) {dim=-3} : f32\nout %1\n", "dim=-1 or dim=-2"),
    ("in %0 : f32[6]\n%1 = sum(%0) {dim=-2} : f32\nout %1\n", "rank"),
    ("in %0 : f32[1,6]\n%1 = var(%0) {dim=-2, correction=1} : f32\nout %1\n", "correction"),
    ("in %0 : f32[4]\n%1 = maximum(%0) : f32\nout %1\n", "takes 2"),
])
def test_ill_formed_graphs_are_compile_errors(text, frag):
    with pytest.raises(pf.PfError) as e:
        pf.Exec(text)
    assert e.value.status == pf.PF_E_COMPILE
    assert frag in str(e.value), str(e.value)


def test_runtime_argument_errors_need_no_gpu():
    e = pf.Exec(configs.cfg3_bias_gelu_gate(rows=4, cols=8).text)
    with pytest.raises(pf.PfError) as err:
        e.execute([16, 32], [64])                                # wrong buffer count
    assert err.value.status == pf.PF_E_RUNTIME
    with pytest.raises(pf.PfError) as err:
        e.execute([16, 32, 0], [64])                             # NULL buffer
    assert err.value.status == pf.PF_E_RUNTIME
    with pytest.raises(pf.PfError) as err:
        e.execute([16, 32, 52], [64])                            # misaligned
    assert err.value.status == pf.PF_E_INVALID
    u = pf.Exec(configs.cfg3_bias_gelu_gate(rows=4, cols=8).text, fuse=False)
    assert u.info()["workspace_bytes"] > 0
    with pytest.raises(pf.PfError) as err:
        u.execute([16, 32, 48], [64], 0, 0)                      # workspace missing
    assert err.value.status == pf.PF_E_RUNTIME


def test_named_subgraphs_fuse_into_one_kernel_and_unfuse_into_one_per_node():
    expect = [(configs.cfg1_add_layernorm(), "row_resident", 10), (configs.cfg2_masked_softmax(heads=1), "row_resident", 7),
              (configs.cfg3_bias_gelu_gate(rows=8), "ew_flat", 3), (configs.cfg4_rmsnorm_rope(1, 8), "row_resident", 10)]
    for w, tmpl, n_ops in expect:
        e = pf.Exec(w.text)
        info = e.info()
        assert info["n_kernels"] == 1 and info["workspace_bytes"] == 0
        assert info["algorithmic_bytes"] == w.algorithmic_bytes == info["planned_bytes"]
        gi = e.group_info(0)
        assert gi["template"] == tmpl and len(gi["nodes"]) == n_ops
        u = pf.Exec(w.text, fuse=False)
        assert u.info()["n_kernels"] == n_ops
        assert u.info()["planned_bytes"] > info["planned_bytes"]


def test_prefix_kernel_count_is_monotone_with_plateaus_inside_groups():
    # K(P): kernels needed for the first P operator nodes.  Inside a fusible run
    # adding an operator adds no kernel (the paper's prefix analysis).
    w = configs.cfg1_add_layernorm()
    lines = w.text.splitlines()
    op_lines = [i for i, l in enumerate(lines) if l.startswith("%") and "const" not in l]
    counts = []
    for p in range(1, len(op_lines) + 1):
        upto = op_lines[p - 1]
        nid = int(lines[upto].split("=")[0].strip()[1:])
        text = "\n".join(l for l in lines[:upto + 1]) + "\nout %%%d\n" % nid
        counts.append(pf.Exec(text).info()["n_kernels"])
    assert counts == [1] * len(counts)
    # a transpose of an elementwise value does not end the run: the consumer's kernel recomputes the value
    # on operands it reads in its own orientation (here the only reader of exp(x) is the transpose, so exp
    # is no longer computed in the input's orientation at all)
    g = Builder()
    x = g.input("f32", (64, 96))
    e = g.op("exp", [x], "f32")
    t = g.op("transpose", [e], "f32")
    h = g.op("tanh", [t], "f32")
    s = g.op("sum", [h], "f32")
    y = g.op("div", [h, s], "f32")
    g.output(y)
    # ... and the row sum of the transposed value is a column sum of tanh(exp(x)) in x's own orientation: no full-size
    # value crosses kernels (x is read twice, y written once, the 96 sums go through memory)
    ex = pf.Exec(g.text())
    assert [gi["template"] for gi in ex.groups()] == ["col_reduce", "tile"]
    assert [gi["nodes"] for gi in ex.groups()] == [[e, h, s], [t, h, y]]
    assert ex.info()["planned_bytes"] == 64 * 96 * 4 * 3 + 2 * 96 * 4
    assert pf.Exec(g.text(), fuse=False).info()["n_kernels"] == 5
    # a per-row statistic changes orientation without moving data: only the statistic itself crosses kernels
    g = Builder()
    x = g.input("f32", (64, 96))
    m = g.op("max", [x], "f32")
    d = g.op("sub", [x, m], "f32")
    t = g.op("transpose", [d], "f32")
    g.output(g.op("exp", [t], "f32"))
    ex = pf.Exec(g.text())
    assert [gi["template"] for gi in ex.groups()] == ["row_resident", "tile"]
    assert ex.info()["workspace_bytes"] == 256 and ex.info()["planned_bytes"] == 64 * 96 * 4 * 3 + 2 * 64 * 4
    # a value of more full-size operands than the round trip through memory would move stays a boundary
    g = Builder()
    ins = [g.input("f32", (64, 96)) for _ in range(4)]
    a = g.op("add", [g.op("add", [ins[0], ins[1]], "f32"), g.op("mul", [ins[2], ins[3]], "f32")], "f32")
    g.output(g.op("exp", [g.op("transpose", [a], "f32")], "f32"))
    ex = pf.Exec(g.text())
    assert [gi["template"] for gi in ex.groups()] == ["ew_flat", "tile"] and ex.info()["workspace_bytes"] == 64 * 96 * 4
    # a value needed in both orientations is computed once, by the tile kernel of the transposed consumer, and stored in
    # its own orientation through that kernel's LDS transpose: x is read once, both results are written once
    g = Builder()
    x = g.input("bf16", (64, 96))
    e = g.op("exp", [x], "bf16")
    g.output(e)
    g.output(g.op("tanh", [g.op("transpose", [e], "bf16")], "bf16"))
    ex = pf.Exec(g.text())
    assert ex.info()["n_kernels"] == 1 and ex.info()["workspace_bytes"] == 0 and ex.group_info(0)["template"] == "tile"
    assert ex.info()["planned_bytes"] == 64 * 96 * 2 * 3


def test_every_random_dag_plans_and_compiles():
    fused_k = unfused_k = ops = 0
    for k in range(0, dags.N_DAGS, 8):
        w = dags.cfg5(k, with_inputs=False)
        f = pf.Exec(w.text)
        fused_k += f.info()["n_kernels"]
        ops += w.meta["n_ops"]
        nodes = [n for gi in f.groups() for n in gi["nodes"]]
        g = pf.Graph(w.text)
        op_ids = {i for i in range(g.size()[0]) if g.node_info(i)["op"] not in ("input", "const")}
        outs = {i for i in op_ids if g.node_info(i)["is_output"]}
        # every reported node is an operator of the graph, every output is computed; a node may be computed
        # twice (once per orientation) or not at all in its own orientation (only a transpose reads it)
        assert set(nodes) <= op_ids and outs <= set(nodes) and len(nodes) <= len(op_ids) + 8
        assert f.info()["algorithmic_bytes"] == w.algorithmic_bytes
    assert fused_k < ops


def test_generated_source_is_inspectable_and_specialised():
    e = pf.Exec(configs.cfg2_masked_softmax(heads=2, seq=512).text)
    src = e.source(0)
    assert 'extern "C" __global__' in src and "pf_team_max" in src and "C = 512" in src
    assert e.group_info(0)["lanes_per_row"] in (16, 32, 64)


def test_keepdim0_reduction_is_read_back_from_memory_by_its_consumers():
    g = Builder()
    x = g.input("f32", (8, 8))
    s = g.op("sum", [x], "f32", keepdim=0)                       # shape [8]: aligns with columns
    y = g.op("add", [x, s], "f32")
    g.output(y)
    e = pf.Exec(g.text())
    assert e.info()["n_kernels"] == 2


def test_roll_and_slice_fold_into_the_consumer():
    w = configs.roll_slice_add_layernorm()
    e = pf.Exec(w.text)
    assert e.info()["n_kernels"] == 1 and e.group_info(0)["template"] == "row_resident"
    assert "% 133" in e.source(0)                                # the roll became index arithmetic
    g = pf.Graph(w.text)
    assert pf.Graph(g.text()).text() == g.text()
    assert g.node_info(7)["shape"] == (128, 128, 96)


@pytest.mark.parametrize("text,frag", [
    ("in %0 : f32[4,6]\n%1 = slice(%0) {dim=1, start=2, stop=7} : f32\nout %1\n", "out of bounds"),
    ("in %0 : f32[4,6]\n%1 = slice(%0) {dim=1, start=3, stop=3} : f32\nout %1\n", "out of bounds"),
    ("in %0 : f32[4,6]\n%1 = roll(%0) {shift=1, dim=2} : f32\nout %1\n", "out of range"),
    ("in %0 : f32[4,6]\n%1 = roll(%0) {dim=1} : f32\nout %1\n", "shift"),
    ("in %0 : f32[4,6]\n%1 = slice(%0) {start=0, stop=2} : f32\nout %1\n", "dim"),
])
def test_ill_formed_views_are_compile_errors(text, frag):
    with pytest.raises(pf.PfError) as e:
        pf.Exec(text)
    assert e.value.status == pf.PF_E_COMPILE and frag in str(e.value)


def test_case_2_pooling_over_the_sequence_dim_is_one_column_reduction_kernel():
    w = configs.masked_mean_pooling(B=4, S=64, D=256)
    e = pf.Exec(w.text)
    assert e.info()["n_kernels"] == 1 and e.info()["workspace_bytes"] == 0
    assert e.info()["planned_bytes"] == w.algorithmic_bytes
    gi = e.group_info(0)
    assert gi["template"] == "col_reduce" and len(gi["nodes"]) == 5
    src = e.source(0)
    assert "S = 64" in src and "DD = 256" in src and "pf_max_nan" in src and "double a" in src    # fp32 output: fp64 accumulators
    assert pf.Exec(w.text, fuse=False).info()["n_kernels"] == 5
    g = pf.Graph(w.text)
    assert "dim=-2" in g.text() and g.node_info(3)["shape"] == (4, 256)
    # few column tiles and many rows: rows split over workgroups, partial sums combined by a second kernel
    sp = pf.Exec(configs.masked_mean_pooling(B=1, S=2048, D=512).text)
    assert sp.info()["n_kernels"] == 2 and len(sp.groups()) == 1 and sp.info()["workspace_bytes"] > 0
    assert "_fin(" in sp.source(0) and "scratch" in sp.source(0)
    with pytest.raises(pf.PfError) as err:
        sp.execute([256, 512], [1024], 0, 0)                         # the partial sums need the workspace
    assert err.value.status == pf.PF_E_RUNTIME
    # a full-shape consumer of the reduced value cannot stay in the kernel
    b = Builder()
    x = b.input("f32", (8, 16))
    m = b.op("mean", [x], "f32", dim=-2, keepdim=1)
    b.output(b.op("sub", [x, m], "f32"))
    assert [gi["template"] for gi in pf.Exec(b.text()).groups()] == ["col_reduce", "ew_flat"]
    # reductions over different dims of the same tensor are different kernels (they need not be different launches:
    # independent of each other, one rides on the other as an extra workgroup)
    b = Builder()
    x = b.input("f32", (8, 16))
    b.output(b.op("sum", [x], "f32", dim=-2))
    b.output(b.op("sum", [x], "f32"))
    both = pf.Exec(b.text())
    assert both.info()["n_kernels"] == 1 and "pf_rider0" in both.source(0)
    assert sorted(gi["template"] for gi in pf.Exec(b.text(), fuse=False).groups()) == ["col_reduce", "row_resident"]


def test_fp16_tensors_parse_print_and_compile():
    w = configs.cfg3_bias_gelu_gate(rows=4, cols=8, dtype="f16")
    g = pf.Graph(w.text)
    assert g.text().count("f16") == 6 and pf.Graph(g.text()).text() == g.text()
    e = pf.Exec(w.text)
    assert e.info()["n_kernels"] == 1 and e.info()["algorithmic_bytes"] == w.algorithmic_bytes == 2 * (4 * 8 * 3 + 8)
    assert "const f16* __restrict__" in e.source(0)
    assert pf.tolerance("f16", -5) == (1e-3, 1e-5) and pf.tolerance("f16", 0) == (1.0, 1.0)


def test_members_that_differ_in_the_outermost_extent_share_one_code_object():
    # Sec. 3.1 task instance: flat and row kernels take the outermost extent as an argument, so
    # members with the same tiling decisions generate the same text (the kernel name ends in its hash)
    g = pf.Graph(configs.cfg3_bias_gelu_gate(rows=4, cols=2048).text)
    execs = [pf.Exec(g.variant([(r, 2048), (2048,), (r, 2048)])) for r in (4, 100, 777)]
    names = {e.kernel_name(0) for e in execs}
    assert len(names) == 1
    src = execs[1].source(0)
    assert "const long long pf_d0" in src and "100" not in src.replace("0x", "")
    assert [e.group_info(0)["grid_blocks"] for e in execs] == [4, 100, 777]      # 2048 bf16 = one 256-lane block per row
    assert execs[0].source(0) == src == execs[2].source(0)
    before = pf.jit_stats()
    again = pf.Exec(g.variant([(900, 2048), (2048,), (900, 2048)]))           # still under the streaming-store threshold
    after = pf.jit_stats()
    assert again.kernel_name(0) in names
    assert after["memory_hits"] == before["memory_hits"] + 1 and after["compiled"] == before["compiled"]
    assert after["code_objects"] == before["code_objects"]
    # another row length is another kernel
    other = pf.Exec(g.variant([(100, 1024), (1024,), (100, 1024)]))
    assert other.kernel_name(0) not in names
    # row kernels: the batch of a softmax; a rank-1 problem has no outer extent to pass
    s = pf.Graph(configs.cfg2_masked_softmax(heads=2, seq=128).text)
    sm = [pf.Exec(s.variant([(h, 128, 128), (128, 128)])) for h in (2, 3, 8)]
    assert len({e.kernel_name(0) for e in sm}) == 1 and "pf_d0" in sm[0].source(0)
    b = Builder()
    b.output(b.op("gelu", [b.input("f32", (1000,))], "f32"))
    assert "pf_d0" not in pf.Exec(b.text()).source(0)


def test_execute_at_another_outer_extent_is_refused_where_the_kernel_is_specialised():
    # argument checks run before anything is enqueued, so they need no GPU
    e = pf.Exec(configs.cfg3_bias_gelu_gate(rows=64, cols=256).text)
    for bad in (0, 65, -3):
        with pytest.raises(pf.PfError) as err:
            e.execute_outer(bad, [16, 16, 16], [16])
        assert err.value.status == pf.PF_E_INVALID and "outermost extent" in str(err.value)
    # a transposing kernel, a two-kernel plan and a rank-1 problem keep every extent literal
    g = Builder()
    x = g.input("f32", (64, 96))
    g.output(g.op("exp", [g.op("transpose", [x], "f32")], "f32"))
    with pytest.raises(pf.PfError) as err:
        pf.Exec(g.text()).execute_outer(32, [16], [16])
    assert "specialised" in str(err.value)
    g = Builder()
    x = g.input("f32", (64, 96))
    s = g.op("sum", [x], "f32", keepdim=0)
    g.output(g.op("exp", [s], "f32"))
    with pytest.raises(pf.PfError) as err:
        pf.Exec(g.text()).execute_outer(32, [16], [16])
    assert err.value.status == pf.PF_E_INVALID
    # a LayerNorm kernel compiled for whole groups of rows wants a multiple of them
    e = pf.Exec(configs.cfg1_add_layernorm(rows=1 << 16, cols=96).text)
    assert e.group_info(0)["template"] == "row_resident"
    if "RU = 1," not in e.source(0):
        with pytest.raises(pf.PfError) as err:
            e.execute_outer(1001, [16, 16, 16, 16], [16])
        assert "multiple" in str(err.value)


def test_many_transposed_operands_stay_within_the_lds_a_workgroup_may_declare():
    # every transposed operand is staged through an LDS tile of its own; the planner stops a tiled group
    # before the tiles outgrow 64 KB and the template narrows its tiles when it has to
    import re
    g = Builder()
    acc = None
    for _ in range(14):
        t = g.op("transpose", [g.input("f32", (4096, 4096))], "f32")
        acc = t if acc is None else g.op("add", [acc, t], "f32")
    g.output(acc)
    e = pf.Exec(g.text())
    assert e.info()["n_kernels"] >= 2                      # 14 tiles do not fit one kernel
    for k, gi in enumerate(e.groups()):
        if gi["template"] != "tile":
            continue
        m = re.search(r"__shared__ float tile\[(\d+)\]\[TS\]\[TS \+ 1\]", e.source(k))
        ts = int(re.search(r"constexpr int TS = (\d+)", e.source(k)).group(1))
        assert m and int(m.group(1)) * ts * (ts + 1) * 4 <= 64 * 1024, (k, m.group(1), ts)


def test_tensors_of_2_to_the_30_elements_and_more_are_indexed_with_64_bits():
    b = Builder()
    x = b.input("bf16", (1 << 15, 1 << 15))
    b.output(b.op("gelu", [x], "bf16"))
    src = pf.Exec(b.text()).source(0)
    assert "const long long e0" in src and "unsigned e0" not in src
    small = Builder()
    small.output(small.op("gelu", [small.input("bf16", (1 << 14, 1 << 15))], "bf16"))
    assert "const unsigned e0" in pf.Exec(small.text()).source(0)
    w = configs.cfg2_masked_softmax(heads=2, seq=512)
    wide = pf.Graph(w.text).variant([(4100, 512, 512), (512, 512)])
    assert "long long grp_raw" in pf.Exec(wide).source(0)


def test_results_too_large_to_index_or_to_launch_are_compile_errors():
    # a broadcast grows far beyond its operands: the result obeys the same size limit as an input
    b = Builder()
    y = b.op("add", [b.input("f32", (1000000, 1000000, 1)), b.input("f32", (1, 1000000))], "f32")
    with pytest.raises(pf.PfError) as err:
        b.output(y)
        pf.Exec(b.text())
    assert err.value.status == pf.PF_E_COMPILE and "too large" in str(err.value)
    # the largest tensors the size limit admits still fit a launch (the library refuses a grid it cannot count)
    b = Builder()
    b.output(b.op("exp", [b.input("bf16", (1 << 20, 1 << 19))], "bf16"))
    assert 0 < pf.Exec(b.text()).group_info(0)["grid_blocks"] < 2 ** 31


def test_cached_code_objects_are_tied_to_the_compiler_and_the_target(tmp_path, monkeypatch):
    import glob
    monkeypatch.setenv("PF_CACHE_DIR", str(tmp_path))
    b = Builder()
    b.output(b.op("tanh", [b.op("exp", [b.input("f32", (37, 53))], "f32")], "f32"))     # a kernel nothing else compiles
    s0 = pf.jit_stats()
    pf.Exec(b.text())
    s1 = pf.jit_stats()
    assert s1["compiled"] == s0["compiled"] + 1
    files = glob.glob(str(tmp_path / "*.pfk"))
    assert len(files) == 1
    blob = open(files[0], "rb").read()
    assert blob[:8] == b"PFCACHE2" and b"gfx950" in blob[24:64] and b"hiprtc" in blob[24:64]
    # the same file under another compiler version is not this compiler's object: it must not be loaded
    tlen = int.from_bytes(blob[8:16], "little")
    forged = bytearray(blob)
    forged[24:24 + tlen] = bytes(blob[24:24 + tlen]).replace(b"hiprtc", b"hiprtC")
    open(files[0], "wb").write(bytes(forged))
    import subprocess, sys
    code = ("import os,sys; sys.path.insert(0, %r); import paper_2605_29357_amd as pf; pf.Exec(%r); s = pf.jit_stats(); "
            "print(s['compiled'], s['disk_hits'])") % (ROOT, b.text())
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=dict(os.environ, PF_CACHE_DIR=str(tmp_path)))
    assert out.stdout.split() == ["1", "0"], out.stdout + out.stderr
    # and once rewritten by this compiler it is a hit for the next process
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=dict(os.environ, PF_CACHE_DIR=str(tmp_path)))
    assert out.stdout.split() == ["0", "1"], out.stdout + out.stderr


def _plan(build, shapes, dtypes):
    g = Builder()
    ins = [g.input(dt, sh) for sh, dt in zip(shapes, dtypes)]
    for o in build(g, ins):
        g.output(o)
    e = pf.Exec(g.text())
    return e, [gi["template"] for gi in e.groups()], e.info()


def test_a_reader_of_a_moved_reduction_joins_the_tile_kernel_that_computes_its_other_operand():
    # y = x * max(x) with x = w / transpose(a): the row maximum of the transposed value is a column maximum in a's own
    # orientation; the product then joins the tile kernel that computes x, although that group was opened
    # before the reduction's (the groups are put in execution order afterwards), so x never crosses memory
    R, C = 96, 200

    def build(g, ins):
        a, wgt = ins                                        # [C, R], [C]
        x = g.op("div", [wgt, g.op("transpose", [a], "f32")], "f32")      # [R, C]
        return [g.op("mul", [x, g.op("max", [x], "f32")], "f32")]

    e, tmpl, info = _plan(build, [(C, R), (C,)], ["f32"] * 2)
    assert tmpl == ["col_reduce", "tile"]
    assert info["planned_bytes"] == 4 * (2 * (R * C + C) + R * C + 2 * R)        # a and w twice, y once, the maxima out and in
    assert info["workspace_bytes"] <= 256 * ((4 * R + 255) // 256)


def test_unrelated_statistics_of_one_tensor_shape_share_a_kernel():
    # sum(a), a transposed output in between, then max(b) - a: the two row statistics have no operand in common when
    # the second is placed, and still run in one row kernel
    R, C = 300, 96

    def build(g, ins):
        a, b = ins
        s = g.op("sum", [a], "f32")
        t = g.op("transpose", [g.op("div", [a, b], "f32")], "f32")
        m = g.op("sub", [a, g.op("max", [b], "f32")], "f32")
        return [s, t, m]

    e, tmpl, info = _plan(build, [(R, C), (R, C)], ["f32"] * 2)
    assert sorted(tmpl) == ["row_resident", "tile"] and info["n_kernels"] == 2


def test_a_16_bit_value_that_is_only_moved_crosses_kernels_in_16_bits():
    # y = tanh(a) * mean(a) lives in a row kernel; its only reader is a transpose that is a bf16 graph output, so the
    # scratch copy is bf16 (rounding before or after the move gives the same bits) instead of fp32
    R, C = 512, 384

    def build(g, ins):
        a, b, c, d = ins
        y = g.op("mul", [g.op("mul", [g.op("mul", [g.op("tanh", [a], "bf16"), g.op("mean", [a], "bf16")], "bf16"), b], "bf16"), c], "bf16")
        return [g.op("transpose", [g.op("mul", [y, d], "bf16")], "bf16"), g.op("max", [a], "bf16")]

    e, tmpl, info = _plan(build, [(R, C)] * 4, ["bf16"] * 4)
    assert tmpl == ["row_resident", "tile"]
    assert info["workspace_bytes"] == 2 * R * C
    # ... but a value that later arithmetic reads stays in fp32
    def build2(g, ins):
        a, b, c, d = ins
        y = g.op("mul", [g.op("mul", [g.op("mul", [g.op("tanh", [a], "bf16"), g.op("mean", [a], "bf16")], "bf16"), b], "bf16"), c], "bf16")
        t = g.op("transpose", [g.op("mul", [y, d], "bf16")], "bf16")
        return [g.op("sum", [t], "bf16"), g.op("max", [a], "bf16")]

    e2, tmpl2, info2 = _plan(build2, [(R, C)] * 4, ["bf16"] * 4)
    assert info2["workspace_bytes"] == 0 or info2["workspace_bytes"] >= 4 * R * C or "col_reduce" in tmpl2


def test_the_tile_edge_can_be_overridden_for_experiments():
    g = Builder()
    x = g.input("f32", (300, 200))
    g.output(g.op("exp", [g.op("transpose", [x], "f32")], "f32"))
    auto = pf.Exec(g.text()).source(0)
    assert "TS = 32" in auto                                     # a small problem: many small tiles
    assert "TS = 64" in pf.Exec(g.text(), tune_tile_edge=64).source(0)
    assert "TS = 32" in pf.Exec(g.text(), tune_tile_edge=32).source(0)
    with pytest.raises(pf.PfError, match="tune_tile_edge"):
        pf.Exec(g.text(), tune_tile_edge=48)


def test_riders_keep_their_pointers_together_in_the_host_signature():
    # two one-workgroup side computations ride on the main kernel: the launch passes, after the host's own arguments,
    # each rider's operands and then its results, rider by rider - the signature must list them in that order
    g = Builder()
    x, wgt, per_row = g.input("f32", (300, 96)), g.input("f32", (96,)), g.input("f32", (300, 1))
    g.output(g.op("mul", [g.op("sub", [x, g.op("mean", [x], "f32")], "f32"), wgt], "f32"))
    g.output(g.op("mul", [g.op("sigmoid", [wgt], "f32"), g.const(2.0, "f32")], "f32"))
    g.output(g.op("sum", [g.op("exp", [wgt], "f32")], "f32"))
    g.output(g.op("tanh", [per_row], "f32"))
    e = pf.Exec(g.text())
    assert e.info()["n_kernels"] == 1
    src = e.source(0)
    sig = src[src.index('extern "C" __global__'):]
    sig = sig[sig.index("(", sig.index(")") + 1) + 1:sig.index(") {")]          # past __launch_bounds__(256)
    names = [p.split()[-1] for p in sig.split(",")]
    own = [n for n in names if not n.startswith("r")]
    riders = [n for n in names if n.startswith("r")]
    assert names == own + riders and own[-1] == "pf_d0"
    assert [n[0] for n in own[:-1]] == sorted(n[0] for n in own[:-1])              # p..., then q...
    # rider by rider, operands before results
    keys = [(int(n[1:n.index("_")]), n[n.index("_") + 1]) for n in riders]
    assert keys == sorted(keys) and {k[0] for k in keys} == {0, 1}
    assert sum(1 for k in keys if k[1] == "q") == 3 and len(own) - 1 == 2 + 1      # three side results; host: x, w in, one out
    # the extra workgroups are dispatched before anything else happens
    body = src[src.index(") {", src.index('extern "C" __global__')):]
    assert body.index("pf_rider0::pf_rider_kernel") < body.index("constexpr int T")
    grid = e.group_info(0)["grid_blocks"]
    assert "blockIdx.x >= %du && blockIdx.x < %du" % (grid - 1, grid) in body and "blockIdx.x >= %du && blockIdx.x < %du" % (grid - 2, grid - 1) in body
