"""torch plumbing around the C ABI: device memory and streams only.

torch allocates the buffers and owns the stream; every computation is done by
libpf.so through the binding in this package.
"""
import ctypes

import numpy as np
import torch

import paper_2605_29357_amd as pf

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64, "f16": torch.float16}


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


def alloc_outputs(w, poison=True):
    """Output buffers pre-filled with NaN so that an element a kernel skips cannot pass
    (the paper's reverse-evaluation rule: never score against stale pool memory)."""
    outs = []
    for dt, shape in zip(w.output_dtypes, w.output_shapes):
        t = torch.empty(tuple(shape) if len(shape) else (), dtype=TORCH_DT[dt], device="cuda")
        if poison:
            t.fill_(float("nan"))
        outs.append(t)
    return outs


class Runner:
    """Compiles a workload's DAG once and runs it on device tensors."""

    def __init__(self, w, fuse=True, intermediates_f32=None, upload=True, **tune):
        self.w = w
        self.exe = pf.Exec(w.text, fuse=fuse, intermediates_f32=intermediates_f32, **tune)
        self.info = self.exe.info()
        ws = self.info["workspace_bytes"]
        # scratch for values that cross kernels; poisoned (NaN bit patterns) so that nothing can rely on its content
        self.ws = torch.full((max(ws, 256),), 255, dtype=torch.uint8, device="cuda") if ws else None
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


_hip = None


def _hiprt():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return _hip


class HipEvent:
    """A raw hipEvent_t (torch's Event hides its handle until it has been recorded)."""

    def __init__(self):
        self._h = ctypes.c_void_p()
        if _hiprt().hipEventCreate(ctypes.byref(self._h)) != 0:
            raise RuntimeError("hipEventCreate failed")
        self.handle = self._h.value

    def record(self, stream):
        if _hiprt().hipEventRecord(self._h, ctypes.c_void_p(stream.cuda_stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_us(self, stop):
        ms = ctypes.c_float()
        if _hiprt().hipEventElapsedTime(ctypes.byref(ms), self._h, stop._h) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value * 1e3

    def __del__(self):
        if _hip is not None and self._h:
            _hip.hipEventDestroy(self._h)
            self._h = None


def score_on_gpu(pairs_spec, stream=None):
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
    ws = torch.full((max(wsb, 256),), 255, dtype=torch.uint8, device="cuda")   # a caller's workspace holds anything: poison it
    s = stream if stream is not None else torch.cuda.current_stream()
    pf.score(pairs, res.data_ptr(), ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    raw = res.cpu().numpy().tobytes()
    return [pf.ScoreResult.from_buffer_copy(raw, i * ctypes.sizeof(pf.ScoreResult)).as_dict() for i in range(n)]


def ladder_on_gpu(pairs_spec, stream=None):
    """pairs_spec: list of (cand_tensor, cand_dtype, ref_tensor, ref_dtype, equal_nan).
    Returns per pair the 11 violation counts for t = -10 .. 0."""
    n = len(pairs_spec)
    pairs = []
    for c, cd, r, rd, en in pairs_spec:
        p = pf.Pair()
        p.d_cand, p.d_ref, p.n = c.data_ptr(), r.data_ptr(), c.numel()
        p.cand_dtype, p.ref_dtype, p.equal_nan = pf.DTYPES[cd], pf.DTYPES[rd], int(en)
        pairs.append(p)
    res = torch.zeros(max(n, 1) * ctypes.sizeof(pf.LadderResult), dtype=torch.uint8, device="cuda")
    ws = torch.full((max(pf.score_ladder_workspace_bytes(n), 256),), 255, dtype=torch.uint8, device="cuda")   # poisoned, as above
    s = stream if stream is not None else torch.cuda.current_stream()
    pf.score_ladder(pairs, res.data_ptr(), ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    raw = res.cpu().numpy().tobytes()
    out = []
    for i in range(n):
        lr = pf.LadderResult.from_buffer_copy(raw, i * ctypes.sizeof(pf.LadderResult))
        out.append((lr.n, list(lr.n_viol)))
    return out
