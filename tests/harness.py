"""GPU-side test helpers: expected values always come from oracle/; the fused
path is always called through the C ABI (paper_2605_29357_amd)."""
import numpy as np

from oracle import dag as oracle_dag
from oracle import score as oracle_score
from tests.device import (Runner, alloc_outputs, check_all_guards, score_on_gpu, to_device,  # noqa: F401
                          to_host_bits)
from workloads import configs


def oracle_outputs(w):
    return oracle_dag.run(w.text, w.inputs)

def check_against_oracle(w, outs, refs=None, rtol=None, atol=None, what=""):
    """Element-by-element |gpu - oracle| <= atol + rtol*|oracle| in fp64; NaN positions must agree."""
    check_all_guards()          # nothing was written outside an output or the workspace
    refs = refs if refs is not None else oracle_outputs(w)
    assert len(outs) == len(refs)
    worst = 0.0
    for k, (o, r, dt) in enumerate(zip(outs, refs, w.output_dtypes)):
        got = oracle_dag.upconvert(to_host_bits(o, dt), dt).reshape(r.shape)
        rt = configs.RTOL[dt] if rtol is None else rtol
        at = configs.ATOL[dt] if atol is None else atol
        nan_r, nan_g = np.isnan(r), np.isnan(got)
        assert np.array_equal(nan_r, nan_g), "%s output %d: NaN pattern differs (%d vs %d)" % (what, k, nan_g.sum(), nan_r.sum())
        ok = ~nan_r
        with np.errstate(invalid="ignore"):
            err = np.abs(got[ok] - r[ok])
            eq = got[ok] == r[ok]
            bound = at + rt * np.abs(r[ok])
            bad = ~(eq | (err <= bound))
        if bad.any():
            i = int(np.argmax(np.where(eq, 0, err - bound)))
            raise AssertionError("%s output %d: %d of %d elements out of tolerance; worst got %r want %r" % (
                what, k, int(bad.sum()), bad.size, got[ok].ravel()[i], r[ok].ravel()[i]))
        if err.size:
            with np.errstate(invalid="ignore", divide="ignore"):
                worst = max(worst, float(np.nanmax(np.where(eq, 0, err / np.maximum(bound, 1e-300)))))
    return worst


def oracle_score_dict(cand_bits, cd, ref_bits, rd, rtol, atol, equal_nan=False):
    return oracle_score.score_pair(cand_bits, cd, ref_bits, rd, rtol, atol, equal_nan)
