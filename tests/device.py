"""torch plumbing for the tests and the benchmark: device memory, streams, and
marshalling of buffers into the C ABI.  No arithmetic of the method lives here
and nothing here touches the CPU oracle.

Buffers a kernel writes (outputs, workspaces) can be allocated between two
guard bands: a few KiB of a known byte pattern directly before and directly
after the payload.  A store that lands outside its buffer (the last partial
vector of a ragged row, the edge of a tile, a column split) changes a band and
check_all_guards() reports it, even when the stray value would never show up
in a comparison of the payload.
"""
import ctypes
import weakref

import numpy as np
import torch

import paper_2605_29357_amd as pf

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64, "f16": torch.float16}

GUARD_BYTES = 4096          # each side; keeps the payload 256-byte aligned
GUARD_BYTE = 0xA5
_guarded = []               # weak references to (raw uint8 tensor) of every live guarded allocation


def guarded_bytes(nbytes, fill=None):
    """A device allocation of nbytes between two guard bands.  Returns (payload, raw): payload is a uint8
    view of exactly nbytes; the trailing band starts at the first byte after it."""
    raw = torch.empty(GUARD_BYTES + nbytes + GUARD_BYTES, dtype=torch.uint8, device="cuda")
    raw[:GUARD_BYTES].fill_(GUARD_BYTE)
    raw[GUARD_BYTES + nbytes:].fill_(GUARD_BYTE)
    payload = raw[GUARD_BYTES:GUARD_BYTES + nbytes]
    if fill is not None:
        payload.fill_(fill)
    _guarded.append((weakref.ref(raw), nbytes))
    return payload, raw


def check_all_guards():
    """Synchronises and verifies the bands of every live guarded allocation; raises on the first damaged one."""
    torch.cuda.synchronize()
    alive = []
    for ref, nbytes in _guarded:
        raw = ref()
        if raw is None:
            continue
        alive.append((ref, nbytes))
        lo = raw[:GUARD_BYTES]
        hi = raw[GUARD_BYTES + nbytes:]
        for name, band in (("before", lo), ("after", hi)):
            bad = (band != GUARD_BYTE).nonzero()
            if bad.numel():
                k = int(bad[0])
                raise AssertionError("a kernel wrote outside its buffer: %d damaged bytes in the band %s a %d-byte buffer, first at offset %d"
                                     % (bad.numel(), name, nbytes, k if name == "after" else k - GUARD_BYTES))
    _guarded[:] = alive
    return len(alive)


def to_device(arr, dtype):
    """Stored numpy bits -> device tensor of the matching torch dtype."""
    if dtype in ("bf16", "f16"):
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(TORCH_DT[dtype])
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def to_host_bits(t, dtype):
    """Device tensor -> stored numpy bits (uint16 for bf16 / fp16, float32/float64 otherwise)."""
    if dtype in ("bf16", "f16"):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def alloc_outputs(w, poison=True, guard=None):
    """Output buffers pre-filled with NaN so that an element a kernel skips cannot pass
    (the paper's reverse-evaluation rule: never score against stale pool memory), each between
    guard bands unless guard=False (guard defaults to poison: timing loops ask for neither)."""
    guard = poison if guard is None else guard
    outs = []
    for dt, shape in zip(w.output_dtypes, w.output_shapes):
        shape = tuple(shape) if len(shape) else ()
        tdt = TORCH_DT[dt]
        if guard:
            n = int(np.prod(shape, dtype=np.int64)) if shape else 1
            payload, raw = guarded_bytes(n * torch.empty(0, dtype=tdt).element_size())
            t = payload.view(tdt).view(shape)
            t._pf_raw = raw                       # keeps the bands alive as long as the view
        else:
            t = torch.empty(shape, dtype=tdt, device="cuda")
        if poison:
            t.fill_(float("nan"))
        outs.append(t)
    return outs


class Runner:
    """Compiles a workload's DAG once and runs it on device tensors."""

    def __init__(self, w, fuse=True, intermediates_f32=None, upload=True, guard=True, **tune):
        self.w = w
        self.exe = pf.Exec(w.text, fuse=fuse, intermediates_f32=intermediates_f32, **tune)
        self.info = self.exe.info()
        ws = self.info["workspace_bytes"]
        # scratch for values that cross kernels; poisoned (NaN bit patterns) so that nothing can rely on its content
        self.ws = None
        if ws:
            if guard:
                self.ws, self._ws_raw = guarded_bytes(max(ws, 256), fill=255)
            else:
                self.ws = torch.full((max(ws, 256),), 255, dtype=torch.uint8, device="cuda")
        self.d_in = [to_device(a, dt) for a, dt in zip(w.inputs, w.input_dtypes)] if upload else None

    def run(self, outs=None, stream=None, events=None):
        """events: optional (start, stop) HipEvent pair bracketing the kernels themselves."""
        outs = outs if outs is not None else alloc_outputs(self.w)
        s = stream if stream is not None else torch.cuda.current_stream()
        self.exe.execute([t.data_ptr() for t in self.d_in], [t.data_ptr() for t in outs],
                         self.ws.data_ptr() if self.ws is not None else 0,
                         self.ws.numel() if self.ws is not None else 0, s.cuda_stream,
                         events[0].handle if events else 0, events[1].handle if events else 0)
        return outs


def make_pairs(pairs_spec, with_tol=True):
    """(cand_tensor, cand_dtype, ref_tensor, ref_dtype[, rtol, atol], equal_nan) tuples -> list of pf.Pair."""
    pairs = []
    for spec in pairs_spec:
        if with_tol:
            c, cd, r, rd, rtol, atol, en = spec
        else:
            c, cd, r, rd, en = spec
            rtol = atol = 0.0
        p = pf.Pair()
        p.d_cand, p.d_ref, p.n = c.data_ptr(), r.data_ptr(), c.numel()
        p.cand_dtype, p.ref_dtype = pf.DTYPES[cd], pf.DTYPES[rd]
        p.rtol, p.atol, p.equal_nan = rtol, atol, int(en)
        pairs.append(p)
    return pairs


def read_structs(buf, cls, n):
    raw = buf.cpu().numpy().tobytes()
    return [cls.from_buffer_copy(raw, i * ctypes.sizeof(cls)) for i in range(n)]


def score_on_gpu(pairs_spec, stream=None):
    """pairs_spec: list of (cand_tensor, cand_dtype, ref_tensor, ref_dtype, rtol, atol, equal_nan).
    Returns a list of dicts read back from the device result structs."""
    n = len(pairs_spec)
    pairs = make_pairs(pairs_spec)
    res, _r = guarded_bytes(max(n, 1) * ctypes.sizeof(pf.ScoreResult), fill=0)
    # a caller's workspace holds anything: poison it
    ws, _w = guarded_bytes(max(pf.score_workspace_bytes(n), 256), fill=255)
    s = stream if stream is not None else torch.cuda.current_stream()
    pf.score(pairs, res.data_ptr(), ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    check_all_guards()
    return [r.as_dict() for r in read_structs(res, pf.ScoreResult, n)]


def ladder_on_gpu(pairs_spec, stream=None):
    """pairs_spec: list of (cand_tensor, cand_dtype, ref_tensor, ref_dtype, equal_nan).
    Returns per pair the 11 violation counts for t = -10 .. 0."""
    n = len(pairs_spec)
    pairs = make_pairs(pairs_spec, with_tol=False)
    res, _r = guarded_bytes(max(n, 1) * ctypes.sizeof(pf.LadderResult), fill=0)
    ws, _w = guarded_bytes(max(pf.score_ladder_workspace_bytes(n), 256), fill=255)   # poisoned, as above
    s = stream if stream is not None else torch.cuda.current_stream()
    pf.score_ladder(pairs, res.data_ptr(), ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    check_all_guards()
    return [(lr.n, list(lr.n_viol)) for lr in read_structs(res, pf.LadderResult, n)]


def score_all_on_gpu(pairs_spec, stream=None):
    """Both results from one pass (pf_score_all): pairs_spec as for score_on_gpu.  Returns (score dicts, ladder tuples)."""
    n = len(pairs_spec)
    pairs = make_pairs(pairs_spec)
    sres, _s = guarded_bytes(max(n, 1) * ctypes.sizeof(pf.ScoreResult), fill=0xEE)
    lres, _l = guarded_bytes(max(n, 1) * ctypes.sizeof(pf.LadderResult), fill=0xEE)
    ws, _w = guarded_bytes(max(pf.score_all_workspace_bytes(n), 256), fill=255)
    s = stream if stream is not None else torch.cuda.current_stream()
    pf.score_all(pairs, sres.data_ptr(), lres.data_ptr(), ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    check_all_guards()
    return ([r.as_dict() for r in read_structs(sres, pf.ScoreResult, n)],
            [(lr.n, list(lr.n_viol)) for lr in read_structs(lres, pf.LadderResult, n)])
