"""GPU parity on the 256 seeded random fusible DAGs.

Each DAG is run fused and op-by-op (one kernel per node, fp32 intermediates),
both are compared with the fp64 oracle element by element, and the fused
output is scored against the op-by-op output by the error kernel, whose result
must equal the oracle scorer's on the same two buffers.
"""
import numpy as np
import pytest
import torch

from tests.harness import (Runner, check_against_oracle, oracle_outputs, oracle_score_dict, score_on_gpu,
                           to_host_bits)
from workloads import configs, dags

pytestmark = pytest.mark.gpu

CHUNK = 16


@pytest.mark.parametrize("first", list(range(0, dags.N_DAGS, CHUNK)))
def test_random_dags(first):
    for k in range(first, min(first + CHUNK, dags.N_DAGS)):
        w = dags.cfg5(k)
        print("dag", k, w.name, flush=True)
        refs = oracle_outputs(w)
        fused = Runner(w, fuse=True)
        outs = fused.run()
        torch.cuda.synchronize()
        check_against_oracle(w, outs, refs=refs, what="%s fused" % w.name)
        unfused = Runner(w, fuse=False, intermediates_f32=True, upload=False)
        unfused.d_in = fused.d_in
        uouts = unfused.run()
        torch.cuda.synchronize()
        check_against_oracle(w, uouts, refs=refs, what="%s unfused" % w.name)
        n_ops = w.meta["n_ops"]
        assert unfused.info["n_kernels"] <= n_ops and fused.info["n_kernels"] <= unfused.info["n_kernels"]
        dt = w.meta["dtype"]
        specs = [(o, dt, u, dt, configs.RTOL[dt], configs.ATOL[dt], False) for o, u in zip(outs, uouts)]
        got = score_on_gpu(specs)
        for o, u, g in zip(outs, uouts, got):
            want = oracle_score_dict(to_host_bits(o, dt), dt, to_host_bits(u, dt), dt, configs.RTOL[dt], configs.ATOL[dt])
            assert g == want, (w.name, g, want)
        del fused, unfused, outs, uouts


def test_random_dags_drawn_from_another_seed():
    """Structures the committed workload never contains: the same generator with another seed, every draw the
    oracle certifies as well conditioned (the rule the committed workload was certified with), fused, against
    the oracle."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location(
        "make_cfg5_attempts", os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "make_cfg5_attempts.py"))
    cert = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(cert)
    checked = 0
    for k in range(0, dags.N_DAGS, 3):
        w = dags.draw_dag(k, 0, seed=101, max_rows=40)
        try:
            cert.check(w)
        except cert.Rejected:
            continue
        print("seed 101 dag", k, w.name, flush=True)
        refs = oracle_outputs(w)
        outs = Runner(w).run()
        torch.cuda.synchronize()
        check_against_oracle(w, outs, refs=refs, what="seed 101 dag %d" % k)
        checked += 1
    assert checked >= 70
