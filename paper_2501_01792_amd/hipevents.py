"""HIP events through ctypes, for timing kernels on the stream they are launched on.

The events are handed to hk_hybrid_decode_attn_marked, which records them between its
kernels; elapsed times are read back here with hipEventElapsedTime.
"""
from __future__ import annotations

import ctypes

_hip = None


def hip():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return _hip


class EventSet:
    """``n`` timing events usable as the ``events`` argument of the marked entry point."""

    def __init__(self, n: int):
        self.n = n
        self.array = (ctypes.c_void_p * n)()
        for i in range(n):
            ev = ctypes.c_void_p()
            rc = hip().hipEventCreate(ctypes.byref(ev))
            if rc != 0:
                raise RuntimeError("hipEventCreate failed: %d" % rc)
            self.array[i] = ev

    def elapsed_ms(self, i: int, j: int) -> float:
        """Milliseconds between event i and event j (both must have completed)."""
        out = ctypes.c_float()
        rc = hip().hipEventElapsedTime(ctypes.byref(out), self.array[i], self.array[j])
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(out.value)

    def destroy(self):
        for i in range(self.n):
            if self.array[i]:
                hip().hipEventDestroy(self.array[i])
                self.array[i] = None
