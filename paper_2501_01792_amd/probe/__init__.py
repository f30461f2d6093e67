"""Measurement aids: what a loop of nothing but fp16 MFMAs sustains on the GPU at hand (the benchmark prints it), and
the rate at which row-major rows stream from HBM for different shapes of one load instruction (``measure read``).

Its own small library (libhkprobe.so, built by ``paper_2501_01792_amd.build``), kept apart from the product
library: it is no operation of the method and synchronises the stream.
"""
from __future__ import annotations

import ctypes
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhkprobe.so")
LT_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhkprobe_lt.so")
_lib = None
_lt_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2501_01792_amd.build` first" % LIB_PATH)
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.hkprobe_mfma_rate.restype = ctypes.c_int
        _lib.hkprobe_mfma_rate.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
        _lib.hkprobe_read_rate.restype = ctypes.c_int
        _lib.hkprobe_read_rate.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    return _lib


def read_rate(buf, rows: int, row_bytes: int, rows_per_load: int, nontemporal: bool, iters: int = 5) -> float:
    """GB/s at which ``rows`` x ``row_bytes`` bytes of the GPU tensor ``buf`` stream when every wavefront owns 32 rows
    and one load instruction covers ``rows_per_load`` rows (8, 4, 2, 1) x 1024 / rows_per_load bytes."""
    import torch
    lib = _load()
    if not buf.is_cuda or buf.numel() * buf.element_size() < rows * row_bytes:
        raise ValueError("buf: a GPU tensor of at least rows * row_bytes bytes")
    sink = torch.zeros(rows // 32 + 64, dtype=torch.int32, device="cuda")
    out = ctypes.c_float()
    st = lib.hkprobe_read_rate(rows_per_load, 1 if nontemporal else 0, ctypes.c_void_p(buf.data_ptr()), rows, row_bytes,
                               ctypes.c_void_p(sink.data_ptr()), iters, ctypes.byref(out),
                               ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise RuntimeError("hkprobe_read_rate failed: %d" % st)
    return float(out.value)


def mfma_rate(random_operands: bool, iters: int = 10000) -> float:
    """Sustained TFLOP/s of back-to-back v_mfma_f32_16x16x32_f16 on every compute unit, with all-zero or random
    fp16 operands (the second is the practical ceiling of an fp16 GEMM on this GPU: the clock drops under
    operand toggling)."""
    import torch
    lib = _load()
    sink = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = ctypes.c_float()
    st = lib.hkprobe_mfma_rate(1 if random_operands else 0, iters, ctypes.c_void_p(sink.data_ptr()), sink.numel(),
                                ctypes.byref(out), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise RuntimeError("hkprobe_mfma_rate failed: %d" % st)
    return float(out.value)


def library_gemm_candidates(a, w, out, max_candidates: int = 32, iters: int = 3, workspace_bytes: int = 512 << 20):
    """Mean milliseconds of each kernel the vendor GEMM library offers for ``out[M, N] = a[M, K] @ w[N, K].T`` (fp16 or
    bf16 GPU tensors, fp32 accumulation), in the library's own order of preference; 0.0 for a candidate it refuses or
    whose workspace does not fit.  libhkprobe_lt.so is a library of its own: only this function loads it."""
    import torch
    global _lt_lib
    if _lt_lib is None:
        if not os.path.exists(LT_LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2501_01792_amd.build` first" % LT_LIB_PATH)
        _lt_lib = ctypes.CDLL(LT_LIB_PATH)
        _lt_lib.hkprobe_library_gemm_candidates.restype = ctypes.c_int
        _lt_lib.hkprobe_library_gemm_candidates.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_float),
            ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
    M, K = a.shape
    N = w.shape[0]
    if not (a.is_cuda and w.is_cuda and out.is_cuda and a.is_contiguous() and w.is_contiguous() and out.is_contiguous()):
        raise ValueError("a, w, out: contiguous GPU tensors")
    if w.shape[1] != K or tuple(out.shape) != (M, N) or not (a.dtype == w.dtype == out.dtype) or a.dtype not in (torch.float16, torch.bfloat16):
        raise ValueError("a [M, K], w [N, K], out [M, N], all fp16 or all bf16")
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda")
    ms = (ctypes.c_float * max_candidates)()
    n = ctypes.c_int32()
    st = _lt_lib.hkprobe_library_gemm_candidates(
        ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(w.data_ptr()), ctypes.c_void_p(out.data_ptr()), M, N, K,
        1 if a.dtype == torch.bfloat16 else 0, ctypes.c_void_p(ws.data_ptr()), workspace_bytes, max_candidates, iters, ms,
        ctypes.byref(n), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise RuntimeError("hkprobe_library_gemm_candidates failed: %d" % st)
    return [float(ms[i]) for i in range(n.value)]
