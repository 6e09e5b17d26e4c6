"""Minimal ctypes view of the HIP runtime: events for timing on a given stream.

torch.cuda.Event only sees torch's current stream and hides its handle until the
first record; the benchmark needs raw hipEvent_t handles it can hand to the library.
"""
from __future__ import annotations

import ctypes

_hip = None


def _rt():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return _hip


def _check(err: int, what: str) -> None:
    if err != 0:
        raise RuntimeError(f"{what} failed with hipError_t {err}")


class Event:
    def __init__(self):
        h = ctypes.c_void_p()
        _check(_rt().hipEventCreate(ctypes.byref(h)), "hipEventCreate")
        self.handle = h.value

    def record(self, stream: int | None) -> None:
        _check(_rt().hipEventRecord(self.handle, stream), "hipEventRecord")

    def synchronize(self) -> None:
        _check(_rt().hipEventSynchronize(self.handle), "hipEventSynchronize")

    def elapsed_ms(self, later: "Event") -> float:
        ms = ctypes.c_float()
        _check(_rt().hipEventElapsedTime(ctypes.byref(ms), self.handle, later.handle), "hipEventElapsedTime")
        return float(ms.value)

    def __del__(self):
        try:
            if self.handle:
                _rt().hipEventDestroy(self.handle)
        except Exception:
            pass
