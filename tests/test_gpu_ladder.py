"""GPU parity of the tolerance-ladder scorer: 11 violation counts per pair, exact."""
import numpy as np
import pytest
import torch

from oracle import metric
from tests.device import ladder_on_gpu, score_all_on_gpu, to_device
from workloads import rng

pytestmark = pytest.mark.gpu


def _noisy(n, cd, rd, seed):
    r = np.random.default_rng(seed)
    base = rng.normal(seed, 0, n)
    # relative errors spread over ten decades so that every level separates some elements
    cand = base * (1 + 10.0 ** r.uniform(-11, 0.5, n) * r.choice([-1, 1], n)) + 10.0 ** r.uniform(-12, -2, n)
    ref = base.copy()
    if n > 100:
        idx = r.choice(n, 12, replace=False)
        cand[idx[:3]] = np.nan
        ref[idx[2:5]] = np.nan
        cand[idx[5]] = np.inf
        ref[idx[5:7]] = np.inf
        ref[idx[7:10]] = 0.0
    store = {"f32": lambda x: x.astype(np.float32), "bf16": rng.round_to_bf16_bits, "f64": lambda x: x.astype(np.float64)}
    return store[cd](cand), store[rd](ref)


def test_ladder_counts_match_the_oracle():
    cases = [(0, "f32", "f32"), (5, "bf16", "bf16"), (1000, "f32", "f64"), (16384, "f32", "f32"), (16385, "bf16", "f32"),
             (300007, "f32", "f32"), (1 << 20, "bf16", "bf16"), (77777, "bf16", "f64"), (4099, "f32", "bf16")]
    specs, wants = [], []
    for k, (n, cd, rd) in enumerate(cases):
        for en in (False, True):
            c, r = _noisy(n, cd, rd, 40 + k)
            dc = to_device(c, cd) if n else torch.empty(0, device="cuda")
            dr = to_device(r, rd) if n else torch.empty(0, device="cuda")
            specs.append((dc, cd, dr, rd, en))
            want = []
            for t in metric.LADDER:
                rt, at = metric.tolerance(cd, t)
                from oracle.score import score_pair
                want.append(score_pair(c, cd, r, rd, rt, at, en)["n_viol"])
            wants.append((n, want))
    got = ladder_on_gpu(specs)
    for (n, cd, rd), g, w in zip([c for c in cases for _ in (0, 1)], got, wants):
        assert g[0] == w[0] and g[1] == w[1], (n, cd, rd, g, w)
    # the counts really do differ between levels
    assert len(set(wants[6][1])) > 5


@pytest.mark.parametrize("cd,rd", [("f32", "f32"), ("bf16", "f32"), ("f32", "bf16"), ("f16", "f32")])
def test_ladder_elements_at_the_edge_of_a_level_are_counted_exactly(cd, rd):
    """Differences placed within a few ulp (and within a few 1e-6) of atol_k + rtol_k |b| for every level:
    what a screen in fp32 cannot settle has to come out of the exact path like the oracle's count."""
    from oracle.score import score_pair
    g = np.random.default_rng(7)
    n_per = 3000
    refs, cands = [], []
    for t in metric.LADDER:
        rt, at = metric.tolerance(cd, t)
        b = g.normal(size=n_per) * 10.0 ** g.uniform(-3, 3, n_per)
        if rd == "bf16":       # the reference as it will be stored, so that the bound below is the one the scorer sees
            b = (rng.round_to_bf16_bits(b).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        else:
            b = b.astype(np.float32).astype(np.float64)
        bound = at + rt * np.abs(b)
        eps = g.choice([-4e-6, -2e-6, -3e-7, -6e-8, 0.0, 6e-8, 3e-7, 2e-6, 4e-6], n_per)
        a = b + g.choice([-1.0, 1.0], n_per) * bound * (1.0 + eps)
        refs.append(b)
        cands.append(a)
    ref64, cand64 = np.concatenate(refs), np.concatenate(cands)
    store = {"f32": lambda x: x.astype(np.float32), "bf16": rng.round_to_bf16_bits, "f16": rng.round_to_f16_bits}
    c, r = store[cd](cand64), store[rd](ref64)
    want = [score_pair(c, cd, r, rd, *metric.tolerance(cd, t), False)["n_viol"] for t in metric.LADDER]
    got = ladder_on_gpu([(to_device(c, cd), cd, to_device(r, rd), rd, False)])[0]
    assert got[0] == c.size and got[1] == want, (got, want)
    assert 0 < want[-1] < want[0] < c.size


def test_one_pass_gives_both_results_and_each_equals_the_oracle():
    """pf_score_all: the single-level result and the eleven ladder counts from one read of every pair, on every
    route (one workgroup per pair, chunks with descriptors by value, chunks with staged descriptors)."""
    from oracle.score import score_pair
    sizes = [0, 5, 8192, 8193, 70001, 300007, 1 << 20, 2500017]
    combos = [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "f64"), ("f16", "f16"), ("f32", "bf16")]
    store = {"f32": lambda x: x.astype(np.float32), "bf16": rng.round_to_bf16_bits, "f16": rng.round_to_f16_bits,
             "f64": lambda x: x.astype(np.float64)}
    for n_pairs in (len(sizes), 60):
        specs, want_s, want_l = [], [], []
        for k in range(n_pairs):
            n = sizes[k % len(sizes)] if n_pairs == len(sizes) else [9000, 100, 40000, 8192, 131073][k % 5]
            cd, rd = combos[k % len(combos)]
            c64, r64 = _noisy(n, "f64", "f64", 700 + k)
            c, r = store[cd](c64), store[rd](r64)
            rtol, atol = [(1e-5, 1e-5), (2e-2, 1e-5), (0.0, 0.0)][k % 3]
            en = bool(k & 1)
            dc = to_device(c, cd) if n else torch.empty(0, device="cuda")
            dr = to_device(r, rd) if n else torch.empty(0, device="cuda")
            specs.append((dc, cd, dr, rd, rtol, atol, en))
            with np.errstate(all="ignore"):
                want_s.append(score_pair(c, cd, r, rd, rtol, atol, en))
                want_l.append((n, [score_pair(c, cd, r, rd, *metric.tolerance(cd, t), en)["n_viol"] for t in metric.LADDER]))
        got_s, got_l = score_all_on_gpu(specs)
        for k in range(n_pairs):
            assert got_s[k] == want_s[k], (n_pairs, k, specs[k][1], specs[k][3], got_s[k], want_s[k])
            assert got_l[k][0] == want_l[k][0] and got_l[k][1] == want_l[k][1], (n_pairs, k, specs[k][1], specs[k][3], got_l[k], want_l[k])
