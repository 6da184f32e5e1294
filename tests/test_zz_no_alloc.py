"""pf_score_static (the scorer with the library's own scratch array, for callers that cannot allocate
device memory) against pf_score on the same pairs: every field must be identical, on two calls in a
row that share the array, the second one smaller than the first."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_29357_amd as pf
from tests.device import guarded_bytes, check_all_guards, make_pairs, read_structs, to_device
from workloads import rng

pytestmark = pytest.mark.gpu


def _specs(sizes, seed):
    combos = [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "f64"), ("f16", "f16")]
    store = {"f32": lambda x: x.astype(np.float32), "bf16": rng.round_to_bf16_bits, "f16": rng.round_to_f16_bits,
             "f64": lambda x: x.astype(np.float64)}
    specs = []
    for k, n in enumerate(sizes):
        cd, rd = combos[k % len(combos)]
        rtol, atol = (2e-2, 1e-5) if cd != "f32" else (1e-5, 1e-5)
        base = rng.normal(seed + k, 0, n)
        noise = rng.normal(seed + k, 1, n)
        cand, ref = base * (1 + noise * rtol) + noise * atol * 0.5, base.copy()
        if n >= 64:
            cand[3] = np.nan
            ref[5] = np.inf
            ref[7] = 0.0
            cand[n // 2] = 1e30
        specs.append((to_device(store[cd](cand), cd), cd, to_device(store[rd](ref), rd), rd, rtol, atol, bool(k & 1)))
    return specs


def _both(specs):
    n = len(specs)
    pairs = make_pairs(specs)
    stream = torch.cuda.current_stream()
    size = n * ctypes.sizeof(pf.ScoreResult)
    res_a, _a = guarded_bytes(size, fill=0xEE)
    res_b, _b = guarded_bytes(size, fill=0xEE)
    ws, _w = guarded_bytes(max(pf.score_workspace_bytes(n), 256), fill=255)
    pf.score(pairs, res_a.data_ptr(), ws.data_ptr(), ws.numel(), stream.cuda_stream)
    pf.score_static(pairs, res_b.data_ptr(), stream.cuda_stream)
    stream.synchronize()
    check_all_guards()
    a = [r.as_dict() for r in read_structs(res_a, pf.ScoreResult, n)]
    b = [r.as_dict() for r in read_structs(res_b, pf.ScoreResult, n)]
    return a, b


def test_static_scratch_scorer_equals_the_workspace_scorer_on_two_calls_in_a_row():
    # first call: every route (one workgroup per pair, staged chunks), several descriptor batches
    first = _specs([1, 100, 8192, 8193, 70001, 131073, 600000, 3000017] + [4000 + 37 * k for k in range(60)], 500)
    a, b = _both(first)
    for k, (x, y) in enumerate(zip(a, b)):
        assert x == y, ("first call, pair %d" % k, x, y)
    assert any(r["n_viol"] for r in a) and any(r["nan_cand"] for r in a)
    # second call, smaller: fewer and shorter pairs, through the scratch the first call left behind
    second = _specs([300000, 9000, 50], 900)
    a2, b2 = _both(second)
    for k, (x, y) in enumerate(zip(a2, b2)):
        assert x == y, ("second call, pair %d" % k, x, y)
    # a third one that takes the route without a staging launch (few mid-size pairs)
    a3, b3 = _both(_specs([20000, 131072], 950))
    assert a3 == b3


def test_static_scratch_scorer_refuses_more_pairs_than_its_array_holds():
    x = torch.zeros(64, device="cuda")
    p = make_pairs([(x, "f32", x, "f32", 0.0, 0.0, False)])[0]
    res = torch.zeros((pf.SCORE_STATIC_MAX_PAIRS + 1) * ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
    with pytest.raises(pf.PfError) as e:
        pf.score_static([p] * (pf.SCORE_STATIC_MAX_PAIRS + 1), res.data_ptr())
    assert e.value.status == pf.PF_E_INVALID
    pf.score_static([p] * pf.SCORE_STATIC_MAX_PAIRS, res.data_ptr())          # the most it takes
    torch.cuda.synchronize()
    got = read_structs(res, pf.ScoreResult, pf.SCORE_STATIC_MAX_PAIRS)
    assert all(r.allclose == 1 and r.n == 64 and r.bit_identical == 1 for r in got)
