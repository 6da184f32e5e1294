"""The calls only enqueue kernels on the caller's stream (no allocation, no memset, no synchronisation),
so a caller can capture them into a HIP graph: launch-bound steps (a 4 us kernel plus its scoring) then
replay without per-kernel launch overhead.  Every replay is checked against the eager result, with eager
work and synchronisations between the replays.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_29357_amd as pf
from tests.harness import Runner, check_against_oracle, oracle_outputs
from workloads import configs

pytestmark = pytest.mark.gpu


def _score_pair_args(cand, ref, dt):
    p = pf.Pair()
    p.d_cand, p.d_ref, p.n = cand.data_ptr(), ref.data_ptr(), cand.numel()
    p.cand_dtype = p.ref_dtype = pf.DTYPES[dt]
    p.rtol, p.atol, p.equal_nan = configs.RTOL[dt], configs.ATOL[dt], 0
    return [p]


@pytest.mark.parametrize("make", [lambda: configs.cfg1_add_layernorm(), lambda: configs.cfg2_masked_softmax(heads=4, seq=512),
                                  lambda: configs.masked_mean_pooling(B=1, S=2048, D=512)])      # the last one runs two kernels
def test_execute_and_score_replay_from_a_captured_graph(make):
    w = make()
    dt = w.output_dtypes[0]
    refs = oracle_outputs(w)
    fused, unfused = Runner(w), Runner(w, fuse=False, intermediates_f32=True)
    eager = fused.run()
    ref_out = unfused.run()
    torch.cuda.synchronize()                       # modules are loaded by the first run: never inside a capture
    check_against_oracle(w, eager, refs=refs, what=w.name)
    res = torch.zeros(ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
    sws = torch.full((max(pf.score_workspace_bytes(1), 256),), 255, dtype=torch.uint8, device="cuda")
    outs = [torch.full_like(t, float("nan")) for t in eager]
    pairs = _score_pair_args(outs[0], ref_out[0], dt)
    pf.score(pairs, res.data_ptr(), sws.data_ptr(), sws.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        fused.run(outs, stream=side)
        pf.score(pairs, res.data_ptr(), sws.data_ptr(), sws.numel(), side.cuda_stream)
    want = None
    for replay in range(4):
        for t in outs:
            t.fill_(float("nan"))                  # eager work between the replays: stale results cannot pass
        res.zero_()
        sws.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, exp in zip(outs, eager):
            assert torch.equal(got.view(torch.uint8), exp.view(torch.uint8)), (w.name, replay)
        r = pf.ScoreResult.from_buffer_copy(res.cpu().numpy().tobytes(), 0).as_dict()
        assert r["n"] == outs[0].numel() and r["nan_cand"] == 0
        if want is None:
            want = r
            # the same numbers as an eager scoring call on the same buffers
            res2 = torch.zeros_like(res)
            pf.score(pairs, res2.data_ptr(), sws.data_ptr(), sws.numel(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert pf.ScoreResult.from_buffer_copy(res2.cpu().numpy().tobytes(), 0).as_dict() == r
        assert r == want, (w.name, replay)
