"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

ctypes front end of the plain-C CPU oracle (``hybridkv_oracle.c``): argument
marshalling only, every number is computed by the C loops.  Inputs are numpy
arrays of any float dtype (fp16 as the GPU path reads them); they are widened
exactly to the oracle's precision (``"f64"`` by default, ``"f32"`` for the
single-precision baseline) before the call.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg import this module.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hybridkv_oracle.c")
_LIB = os.path.join(_HERE, "libhybridkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over rows / sequences, no fast-math)."""
    deps = [_SRC, os.path.join(_HERE, "hybridkv_oracle_impl.h")]
    stale = force or not os.path.exists(_LIB) or any(
        os.path.getmtime(p) > os.path.getmtime(_LIB) for p in deps)
    if stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.hko_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loops use on this machine."""
    return int(_load().hko_num_threads())


_PREC = {"f64": (np.float64, ctypes.c_double), "f32": (np.float32, ctypes.c_float)}


def _arr(a, np_t):
    return np.ascontiguousarray(np.asarray(a), dtype=np_t)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def layernorm(x, gamma, beta, eps=1e-5, precision="f64"):
    """LayerNorm of the rows of ``x[M, d]`` -> ``xhat[M, d]``."""
    np_t, c_t = _PREC[precision]
    x = _arr(x, np_t)
    M, d = x.shape
    gamma, beta = _arr(gamma, np_t), _arr(beta, np_t)
    assert gamma.shape == (d,) and beta.shape == (d,)
    out = np.empty_like(x)
    fn = getattr(_load(), "hko_layernorm_" + precision)
    fn(_ptr(x), _ptr(gamma), _ptr(beta), _i64(M), _i64(d), c_t(eps), _ptr(out))
    return out


def kv_projection(xhat, Wkv, bkv, precision="f64"):
    """Eq. 7 plus biases: ``xhat[M, d]``, ``Wkv[N, d]``, ``bkv[N]`` -> ``KV[M, N]``
    (N = 2d for the full fused weight; any subset of its rows gives those features only)."""
    np_t, _ = _PREC[precision]
    xhat = _arr(xhat, np_t)
    M, d = xhat.shape
    Wkv, bkv = _arr(Wkv, np_t), _arr(bkv, np_t)
    N = Wkv.shape[0]
    assert Wkv.shape == (N, d) and bkv.shape == (N,)
    out = np.empty((M, N), dtype=np_t)
    fn = getattr(_load(), "hko_kv_projection_" + precision)
    fn(_ptr(xhat), _ptr(Wkv), _ptr(bkv), _i64(M), _i64(d), _i64(N), _ptr(out))
    return out


def regen_kv(act, gamma, beta, Wkv, bkv, n_heads, eps=1e-5, precision="f64"):
    """KV Gen: ``act[B, L_act, d]`` -> ``(K, V)`` each ``[B, H, L_act, dh]``."""
    np_t, c_t = _PREC[precision]
    act = _arr(act, np_t)
    B, L_act, d = act.shape
    assert d % n_heads == 0
    dh = d // n_heads
    gamma, beta, Wkv, bkv = (_arr(a, np_t) for a in (gamma, beta, Wkv, bkv))
    assert Wkv.shape == (2 * d, d) and bkv.shape == (2 * d,)
    K = np.empty((B, n_heads, L_act, dh), dtype=np_t)
    V = np.empty_like(K)
    s_x = np.empty((B * L_act, d), dtype=np_t)
    s_kv = np.empty((B * L_act, 2 * d), dtype=np_t)
    fn = getattr(_load(), "hko_regen_kv_" + precision)
    fn(_ptr(act), _ptr(gamma), _ptr(beta), _ptr(Wkv), _ptr(bkv),
       _i64(B), _i64(L_act), _i64(d), _i64(n_heads), c_t(eps),
       _ptr(K), _ptr(V), _i64(L_act), _i64(0), _ptr(s_x), _ptr(s_kv))
    return K, V


def decode_attention(q, K, V, scale=None, return_probs=False, precision="f64"):
    """Eq. 4 for one query per (sequence, head): ``q[B,H,dh]``, ``K,V[B,H,L,dh]`` -> ``out[B,H,dh]``."""
    np_t, c_t = _PREC[precision]
    q, K, V = _arr(q, np_t), _arr(K, np_t), _arr(V, np_t)
    B, H, dh = q.shape
    L = K.shape[2]
    assert K.shape == (B, H, L, dh) and V.shape == K.shape
    if scale is None:
        scale = dh ** -0.5
    out = np.empty((B, H, dh), dtype=np_t)
    probs = np.empty((B, H, L), dtype=np_t) if return_probs else None
    fn = getattr(_load(), "hko_decode_attention_" + precision)
    fn(_ptr(q), _ptr(K), _ptr(V), _i64(B), _i64(H), _i64(L), _i64(dh), c_t(scale),
       _ptr(out), _ptr(probs) if return_probs else None)
    return (out, probs) if return_probs else out


def hybrid_decode_attn(q, K_cache, V_cache, act, gamma, beta, Wkv, bkv, n_heads,
                       eps=1e-5, scale=None, precision="f64"):
    """The whole step.  ``K_cache, V_cache[B,H,L_kv,dh]`` (``None`` when L_kv == 0),
    ``act[B,L_act,d]`` (``None`` when L_act == 0).  Returns ``(out[B,H,dh],
    K_full, V_full)`` with ``K_full, V_full[B,H,L_kv+L_act,dh]``."""
    np_t, c_t = _PREC[precision]
    q = _arr(q, np_t)
    B, H, dh = q.shape
    assert H == n_heads
    d = H * dh
    gamma, beta, Wkv, bkv = (_arr(a, np_t) for a in (gamma, beta, Wkv, bkv))
    assert Wkv.shape == (2 * d, d) and bkv.shape == (2 * d,)
    if K_cache is None:
        K_cache = np.zeros((B, H, 0, dh), dtype=np_t)
        V_cache = np.zeros((B, H, 0, dh), dtype=np_t)
    if act is None:
        act = np.zeros((B, 0, d), dtype=np_t)
    K_cache, V_cache, act = _arr(K_cache, np_t), _arr(V_cache, np_t), _arr(act, np_t)
    L_kv, L_act = K_cache.shape[2], act.shape[1]
    assert K_cache.shape == (B, H, L_kv, dh) and V_cache.shape == K_cache.shape
    assert act.shape == (B, L_act, d)
    if scale is None:
        scale = dh ** -0.5
    L = L_kv + L_act
    out = np.empty((B, H, dh), dtype=np_t)
    K_full = np.empty((B, H, L, dh), dtype=np_t)
    V_full = np.empty_like(K_full)
    s_x = np.empty((max(B * L_act, 1), d), dtype=np_t)
    s_kv = np.empty((max(B * L_act, 1), 2 * d), dtype=np_t)
    fn = getattr(_load(), "hko_hybrid_decode_attn_" + precision)
    fn(_ptr(q), _ptr(K_cache), _ptr(V_cache), _i64(L_kv), _ptr(act), _i64(L_act),
       _ptr(gamma), _ptr(beta), _ptr(Wkv), _ptr(bkv),
       _i64(B), _i64(d), _i64(n_heads), c_t(eps), c_t(scale),
       _ptr(out), _ptr(K_full), _ptr(V_full), _ptr(s_x), _ptr(s_kv))
    return out, K_full, V_full


def qkv_current(x_cur, gamma, beta, Wq, bq, Wkv, bkv, n_heads, eps=1e-5, precision="f64"):
    """QKV generation of the current input token of every sequence (Sec. 4.2.2; Eq. 2 with the
    layer's pre-attention LayerNorm in front, biases added): ``x_cur[B, d]`` ->
    ``(q, k, v)``, each ``[B, H, dh]``.  LayerNorm and projection are the routines above: the
    query weight is one more set of output features of the same affine map."""
    x_cur = np.asarray(x_cur)
    B, d = x_cur.shape
    dh = d // n_heads
    xhat = layernorm(x_cur, gamma, beta, eps, precision)
    q = kv_projection(xhat, Wq, bq, precision)
    kv = kv_projection(xhat, Wkv, bkv, precision)
    return (q.reshape(B, n_heads, dh), kv[:, :d].reshape(B, n_heads, dh), kv[:, d:].reshape(B, n_heads, dh))
