"""Tensors of 2^30 elements and more: the generated kernels switch every index to 64 bits there.

The oracle cannot evaluate a billion elements in a test, and need not: every row of these subgraphs
is independent, so it evaluates whole sampled rows (first, last, and the rows around element 2^30)
as a smaller instance of the same DAG; the rest of the output is checked to be written.  The scorer
is checked on the same buffers: differences planted at known positions beyond element 2^30, everything
else identical, so its exact result is the oracle's result on the planted elements alone.

Inputs are drawn on the device from a seeded generator (a billion values from the host generator
would take minutes); the sampled rows the oracle sees are copied back from those same buffers.
"""
import numpy as np
import pytest
import torch

import paper_2605_29357_amd as pf
from oracle import dag as oracle_dag
from tests.device import alloc_outputs, check_all_guards, guarded_bytes, score_on_gpu, to_host_bits
from tests.harness import oracle_score_dict
from workloads import configs

pytestmark = pytest.mark.gpu


def _rows_check(got_rows, ref, dt, what):
    got = oracle_dag.upconvert(got_rows, dt).reshape(ref.shape)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), what
    err = np.abs(got - ref)
    bound = configs.ATOL[dt] + configs.RTOL[dt] * np.abs(ref)
    bad = ~((got == ref) | (err <= bound))
    assert not bad.any(), "%s: %d elements out of tolerance" % (what, int(bad.sum()))


def _run(exe, ins, outs):
    info = exe.info()
    assert info["workspace_bytes"] == 0
    exe.execute([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    check_all_guards()


def test_elementwise_subgraph_beyond_2_to_the_30_elements():
    rows, cols = 97600, 11008                      # 1,074,380,800 elements: element 2^30 lies in row 97541
    assert rows * cols >= 1 << 30
    small = configs.cfg3_bias_gelu_gate(rows=4, cols=cols)
    g = pf.Graph(small.text).variant([(rows, cols), (cols,), (rows, cols)])
    exe = pf.Exec(g)
    assert "long long" in exe.source(0) and exe.group_info(0)["template"] == "ew_flat"
    gen = torch.Generator(device="cuda").manual_seed(41)
    a = torch.randn((rows, cols), device="cuda", dtype=torch.bfloat16, generator=gen)
    b = torch.randn((rows, cols), device="cuda", dtype=torch.bfloat16, generator=gen)
    bias = (0.02 * torch.randn((cols,), device="cuda", generator=gen)).to(torch.bfloat16)
    w = configs.Workload("wide_gate", g.text(), None, ["bf16"] * 3, [(rows, cols), (cols,), (rows, cols)], ["bf16"], [(rows, cols)])
    out = alloc_outputs(w)[0]
    _run(exe, [a, bias, b], [out])
    assert not torch.isnan(out).any()              # every element written (the buffer starts as NaN)
    ids = np.array([0, 1, 48000, 97540, 97541, 97542, rows - 2, rows - 1])
    tid = torch.from_numpy(ids).cuda()
    s = configs.cfg3_bias_gelu_gate(rows=len(ids), cols=cols)
    s.inputs = [to_host_bits(a[tid], "bf16"), to_host_bits(bias, "bf16"), to_host_bits(b[tid], "bf16")]
    ref = oracle_dag.run(s.text, s.inputs)[0]
    _rows_check(to_host_bits(out[tid], "bf16"), ref, "bf16", "wide elementwise")

    # the scorer on the same buffers: out against a copy with differences planted beyond element 2^30
    cand = out.clone()
    flat_c, flat_r = cand.view(-1), out.view(-1)
    n = flat_c.numel()
    pos = torch.tensor([(1 << 30) + 5, (1 << 30) + 8191, n - 1, n - 16385, 12345], device="cuda")
    flat_c[pos] = flat_r[pos] * 1.5 + 3.0
    flat_c[(1 << 30) + 77] = float("nan")
    got = score_on_gpu([(cand, "bf16", out, "bf16", 2e-2, 1e-5, False)])[0]
    sel = torch.cat([pos, torch.tensor([(1 << 30) + 77], device="cuda")])
    want = oracle_score_dict(to_host_bits(flat_c[sel], "bf16"), "bf16", to_host_bits(flat_r[sel], "bf16"), "bf16", 2e-2, 1e-5)
    want["n"] = n
    want["bit_identical"] = 0
    assert got == want, (got, want)
    assert got["n_viol"] == 6 and got["nan_cand"] == 1


def test_row_reduction_subgraph_beyond_2_to_the_30_elements():
    heads, seq = 4100, 512                          # 1,074,790,400 elements; element 2^30 lies in head 4096, row 0
    small = configs.cfg2_masked_softmax(heads=2, seq=seq)
    g = pf.Graph(small.text).variant([(heads, seq, seq), (seq, seq)])
    exe = pf.Exec(g)
    assert "long long" in exe.source(0) and exe.group_info(0)["template"] == "row_resident"
    gen = torch.Generator(device="cuda").manual_seed(43)
    z = (2.0 * torch.randn((heads, seq, seq), device="cuda", generator=gen, dtype=torch.float32)).to(torch.bfloat16)
    mask = torch.from_numpy(configs.causal_mask_bits(seq, "bf16").view(np.int16)).cuda().view(torch.bfloat16)
    w = configs.Workload("wide_softmax", g.text(), None, ["bf16"] * 2, [(heads, seq, seq), (seq, seq)], ["bf16"], [(heads, seq, seq)])
    out = alloc_outputs(w)[0]
    _run(exe, [z, mask], [out])
    assert not torch.isnan(out).any()
    ids = np.array([0, 2047, 4095, 4096, 4097, heads - 1])
    tid = torch.from_numpy(ids).cuda()
    s = configs.cfg2_masked_softmax(heads=len(ids), seq=seq)
    s.inputs = [to_host_bits(z[tid], "bf16"), small.inputs[1]]
    ref = oracle_dag.run(s.text, s.inputs)[0]
    _rows_check(to_host_bits(out[tid], "bf16"), ref, "bf16", "wide softmax")
    # rows sum to one everywhere (a property that holds at any size), masked entries are exactly zero
    sums = out.float().sum(dim=-1)
    assert float((sums - 1).abs().max()) < 2e-2
    assert float(out[:, 0, 1:].abs().max()) == 0.0
