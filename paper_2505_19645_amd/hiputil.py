"""Raw HIP events through ctypes, for timing stages on the stream the kernels
run on.  Plumbing only."""
from __future__ import annotations

import ctypes as C

_hip = None


def hip():
    global _hip
    if _hip is None:
        import torch  # noqa: F401  (loads the process's one HIP runtime)
        _hip = C.CDLL("libamdhip64.so.7")
        _hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
        _hip.hipEventSynchronize.argtypes = [C.c_void_p]
        _hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    return _hip


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with hipError {rc}")


class Event:
    def __init__(self):
        h = C.c_void_p()
        _check(hip().hipEventCreate(C.byref(h)), "hipEventCreate")
        self.handle = h.value

    def record(self, stream_handle: int):
        _check(hip().hipEventRecord(self.handle, stream_handle), "hipEventRecord")

    def synchronize(self):
        _check(hip().hipEventSynchronize(self.handle), "hipEventSynchronize")

    def elapsed_ms(self, later: "Event") -> float:
        ms = C.c_float()
        _check(hip().hipEventElapsedTime(C.byref(ms), self.handle, later.handle), "hipEventElapsedTime")
        return ms.value

    def __del__(self):
        try:
            hip().hipEventDestroy(self.handle)
        except Exception:
            pass
