"""Raw hipEvent_t handles for timing kernels on a caller's stream.

torch's Event hides its handle until it has been recorded, and pf_execute_timed
attaches events to the dispatch itself, so the benchmark and the tests create
their events through the HIP runtime directly.
"""
import ctypes

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
