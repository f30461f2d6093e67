"""Measurement aid of the benchmark: what a loop of nothing but fp16 MFMAs sustains on the GPU at hand.

Its own small library (libhkprobe.so, built by ``paper_2501_01792_amd.build``), kept apart from the product
library: it is no operation of the method and synchronises the stream.
"""
from __future__ import annotations

import ctypes
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhkprobe.so")
_lib = None


def mfma_rate(random_operands: bool, iters: int = 10000) -> float:
    """Sustained TFLOP/s of back-to-back v_mfma_f32_16x16x32_f16 on every compute unit, with all-zero or random
    fp16 operands (the second is the practical ceiling of an fp16 GEMM on this GPU: the clock drops under
    operand toggling)."""
    import torch
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2501_01792_amd.build` first" % LIB_PATH)
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.hkprobe_mfma_rate.restype = ctypes.c_int
        _lib.hkprobe_mfma_rate.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    sink = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = ctypes.c_float()
    st = _lib.hkprobe_mfma_rate(1 if random_operands else 0, iters, ctypes.c_void_p(sink.data_ptr()), sink.numel(),
                                ctypes.byref(out), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise RuntimeError("hkprobe_mfma_rate failed: %d" % st)
    return float(out.value)
