"""GPU-side test helpers: torch owns device memory and the stream, nothing else.

The fused path is always called through the C ABI (paper_2605_29357_amd);
expected values always come from oracle/.
"""
import ctypes

import numpy as np
import torch

import paper_2605_29357_amd as pf
from oracle import dag as oracle_dag
from oracle import score as oracle_score
from workloads import configs

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64}
POISON = {"f32": 0x7FC00000, "bf16": 0x7FC0}


def to_device(arr, dtype):
    """Stored numpy bits -> device tensor of the matching torch dtype."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def to_host_bits(t, dtype):
    """Device tensor -> stored numpy bits (uint16 for bf16, float32/float64 otherwise)."""
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def alloc_outputs(w, poison=True):
    """Output buffers pre-filled with NaN so that an element the kernel skips cannot pass."""
    outs = []
    for dt, shape in zip(w.output_dtypes, w.output_shapes):
        t = torch.empty(tuple(shape) if len(shape) else (), dtype=TORCH_DT[dt], device="cuda")
        if poison:
            t.fill_(float("nan"))
        outs.append(t)
    return outs


class Runner:
    """Compiles a workload's DAG once and runs it on device tensors."""

    def __init__(self, w, fuse=True, intermediates_f32=None):
        self.w = w
        self.exe = pf.Exec(w.text, fuse=fuse, intermediates_f32=intermediates_f32)
        self.info = self.exe.info()
        ws = self.info["workspace_bytes"]
        self.ws = torch.empty(max(ws, 256), dtype=torch.uint8, device="cuda") if ws else None
        self.d_in = [to_device(a, dt) for a, dt in zip(w.inputs, w.input_dtypes)]

    def run(self, outs=None, stream=None):
        outs = outs if outs is not None else alloc_outputs(self.w)
        s = stream if stream is not None else torch.cuda.current_stream()
        self.exe.execute([t.data_ptr() for t in self.d_in], [t.data_ptr() for t in outs],
                         self.ws.data_ptr() if self.ws is not None else 0,
                         self.ws.numel() if self.ws is not None else 0, s.cuda_stream)
        return outs


def oracle_outputs(w):
    return oracle_dag.run(w.text, w.inputs)


def check_against_oracle(w, outs, refs=None, rtol=None, atol=None, what=""):
    """Element-by-element |gpu - oracle| <= atol + rtol*|oracle| in fp64; NaN positions must agree."""
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


def score_on_gpu(pairs_spec):
    """pairs_spec: list of (cand_tensor, cand_dtype, ref_tensor, ref_dtype, rtol, atol, equal_nan).
    Returns a list of dicts read back from the device result structs."""
    n = len(pairs_spec)
    pairs = []
    for c, cd, r, rd, rtol, atol, en in pairs_spec:
        p = pf.Pair()
        p.d_cand, p.d_ref, p.n = c.data_ptr(), r.data_ptr(), c.numel()
        p.cand_dtype, p.ref_dtype = pf.DTYPES[cd], pf.DTYPES[rd]
        p.rtol, p.atol, p.equal_nan = rtol, atol, int(en)
        pairs.append(p)
    res = torch.zeros(max(n, 1) * ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
    wsb = pf.score_workspace_bytes(n)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    pf.score(pairs, res.data_ptr(), ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = res.cpu().numpy().tobytes()
    out = []
    for i in range(n):
        sr = pf.ScoreResult.from_buffer_copy(raw, i * ctypes.sizeof(pf.ScoreResult))
        out.append(sr.as_dict())
    return out


def oracle_score_dict(cand_bits, cd, ref_bits, rd, rtol, atol, equal_nan=False):
    return oracle_score.score_pair(cand_bits, cd, ref_bits, rd, rtol, atol, equal_nan)
