"""ctypes binding of libhybridkv.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's
HIP kernels.  There is no fallback: if the library cannot be loaded the import of a symbol
raises, and a call with a non-GPU tensor raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhybridkv.so")

HK_OK = 0
HK_ERR_NULL, HK_ERR_SHAPE, HK_ERR_RATIO, HK_ERR_ALIGN = -1, -2, -3, -4
HK_ERR_WORKSPACE, HK_ERR_DTYPE, HK_ERR_LAUNCH, HK_ERR_STATIC_LIMIT = -5, -6, -7, -8
HK_STATIC_SCRATCH_BYTES = 32 << 20
HK_DTYPE_F16 = 0
HK_DTYPE_BF16 = 1
HK_MAX_SPLITS = 64


class hk_shape(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("ln_eps", ctypes.c_float), ("softmax_scale", ctypes.c_float),
                ("attn_splits", ctypes.c_int32), ("gemm_tile", ctypes.c_int32)]


class hk_line(ctypes.Structure):
    _fields_ = [("slope", ctypes.c_double), ("offset", ctypes.c_double)]


class hk_alloc_params(ctypes.Structure):
    _fields_ = [("T_load_w", ctypes.c_double), ("T_kv_gen", hk_line), ("T_load_kv", hk_line),
                ("n_act_gpu", ctypes.c_double), ("M_host", ctypes.c_double), ("S_weight", ctypes.c_double),
                ("S_kv", ctypes.c_double)]


class hk_alloc_result(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in ("act_init", "kv_init", "act_remain", "kv_remain", "act_host", "kv_host")]


HK_BLOCK_KV, HK_BLOCK_ACT = 0, 1


class hk_paged_cache(ctypes.Structure):
    _fields_ = [("K_pool", ctypes.c_void_p), ("V_pool", ctypes.c_void_p), ("act_pool", ctypes.c_void_p),
                ("block_table", ctypes.c_void_p), ("seq_len", ctypes.c_void_p), ("cu_tokens", ctypes.c_void_p),
                ("total_tokens", ctypes.c_int64), ("P_kv", ctypes.c_int32), ("P_act", ctypes.c_int32),
                ("n_act_used", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("max_blocks", ctypes.c_int32)]


class hk_layer_params(ctypes.Structure):
    _fields_ = [("ln_w", ctypes.c_void_p), ("ln_b", ctypes.c_void_p),
                ("Wkv", ctypes.c_void_p), ("bkv", ctypes.c_void_p), ("prepared", ctypes.c_void_p)]


class HybridKVError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built (no silent fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2501_01792_amd.build` "
                               "(or __graft_entry__.build()) first" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        shp, lpp = ctypes.POINTER(hk_shape), ctypes.POINTER(hk_layer_params)
        L.hk_workspace_bytes.restype = sz
        L.hk_workspace_bytes.argtypes = [shp, i32, i32, i32]
        L.hk_regen_workspace_bytes.restype = sz
        L.hk_regen_workspace_bytes.argtypes = [shp, i32, i32]
        L.hk_prepared_bytes.restype = sz
        L.hk_prepared_bytes.argtypes = [shp]
        L.hk_prepare_layer.restype = ctypes.c_int
        L.hk_prepare_layer.argtypes = [shp, lpp, vp, sz, vp]
        L.hk_regen_kv.restype = ctypes.c_int
        L.hk_regen_kv.argtypes = [shp, vp, i32, i32, lpp, vp, vp, i32, i32, vp, sz, vp]
        L.hk_hybrid_decode_attn.restype = ctypes.c_int
        L.hk_hybrid_decode_attn.argtypes = [shp, vp, vp, vp, i32, vp, i32, i32, lpp, ctypes.c_float,
                                            vp, vp, sz, vp]
        L.hk_hybrid_decode_attn_marked.restype = ctypes.c_int
        L.hk_hybrid_decode_attn_marked.argtypes = L.hk_hybrid_decode_attn.argtypes + [ctypes.POINTER(vp), i32]
        L.hk_hybrid_decode_attn_static.restype = ctypes.c_int
        L.hk_hybrid_decode_attn_static.argtypes = [shp, vp, vp, vp, i32, vp, i32, i32, lpp, ctypes.c_float, vp, vp]
        L.hk_two_stream_workspace_bytes.restype = sz
        L.hk_two_stream_workspace_bytes.argtypes = [shp, i32, i32, i32]
        L.hk_hybrid_decode_attn_two_stream.restype = ctypes.c_int
        L.hk_hybrid_decode_attn_two_stream.argtypes = [shp, vp, vp, vp, i32, vp, i32, i32, lpp, ctypes.c_float, vp, vp, sz,
                                                       vp, vp, vp, vp, i32]
        L.hk_absorbed_workspace_bytes.restype = sz
        L.hk_absorbed_workspace_bytes.argtypes = [shp, i32, i32, i32]
        L.hk_hybrid_decode_attn_absorbed.restype = ctypes.c_int
        L.hk_hybrid_decode_attn_absorbed.argtypes = L.hk_hybrid_decode_attn.argtypes
        L.hk_qkv_workspace_bytes.restype = ctypes.c_size_t
        L.hk_qkv_workspace_bytes.argtypes = [ctypes.POINTER(hk_shape), i32]
        L.hk_qkv_current.restype = ctypes.c_int
        L.hk_qkv_current.argtypes = [ctypes.POINTER(hk_shape), vp, i32, ctypes.POINTER(hk_layer_params), vp, vp,
                                     vp, vp, vp, i32, i32, vp, i32, i32, vp, sz, vp]
        L.hk_paged_workspace_bytes.restype = ctypes.c_size_t
        L.hk_paged_workspace_bytes.argtypes = [ctypes.POINTER(hk_shape), i32, ctypes.POINTER(hk_paged_cache)]
        L.hk_paged_decode_attn.restype = ctypes.c_int
        L.hk_paged_decode_attn.argtypes = [ctypes.POINTER(hk_shape), vp, i32, ctypes.POINTER(hk_paged_cache),
                                           ctypes.POINTER(hk_layer_params), vp, vp, sz, vp]
        L.hk_paged_absorbed_workspace_bytes.restype = sz
        L.hk_paged_absorbed_workspace_bytes.argtypes = L.hk_paged_workspace_bytes.argtypes
        L.hk_paged_decode_attn_absorbed.restype = ctypes.c_int
        L.hk_paged_decode_attn_absorbed.argtypes = L.hk_paged_decode_attn.argtypes
        L.hk_paged_append.restype = ctypes.c_int
        L.hk_paged_append.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_int64, ctypes.c_int64, vp]
        L.hk_qkv_current_paged.restype = ctypes.c_int
        L.hk_qkv_current_paged.argtypes = [ctypes.POINTER(hk_shape), vp, i32, ctypes.POINTER(hk_layer_params), vp, vp, vp,
                                           ctypes.POINTER(hk_paged_cache), vp, vp, sz, vp]
        dp = ctypes.POINTER(ctypes.c_double)
        L.hk_fit_line.restype = ctypes.c_int
        L.hk_fit_line.argtypes = [dp, dp, i32, ctypes.POINTER(hk_line), dp]
        L.hk_host_block_allocation.restype = ctypes.c_int
        L.hk_host_block_allocation.argtypes = [ctypes.POINTER(hk_alloc_params), ctypes.POINTER(hk_alloc_result)]
        L.hk_next_block_type.restype = ctypes.c_int
        L.hk_next_block_type.argtypes = [ctypes.c_int64] * 4
        L.hk_minibatch_balance.restype = ctypes.c_int
        L.hk_minibatch_balance.argtypes = [ctypes.POINTER(hk_line), ctypes.POINTER(hk_line), ctypes.c_double,
                                           ctypes.c_double, dp, dp]
        L.hk_regen_offsets.restype = ctypes.c_int
        L.hk_regen_offsets.argtypes = [shp, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.hk_status_string.restype = ctypes.c_char_p
        L.hk_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hk_status_string(int(status)).decode()


def make_shape(d, n_heads, ln_eps=1e-5, softmax_scale=0.0, attn_splits=0, gemm_tile=0, dtype=HK_DTYPE_F16) -> hk_shape:
    return hk_shape(d, n_heads, d // n_heads, dtype, ln_eps, softmax_scale, attn_splits, gemm_tile)


def _dtype_code(t):
    """The C ABI's dtype code of a tensor: fp16, or bf16 where the entry point takes it."""
    import torch
    return HK_DTYPE_BF16 if t.dtype == torch.bfloat16 else HK_DTYPE_F16


def hk_workspace_bytes(shape: hk_shape, B: int, L_kv: int, L_act: int) -> int:
    return int(lib().hk_workspace_bytes(ctypes.byref(shape), B, L_kv, L_act))


def hk_regen_workspace_bytes(shape: hk_shape, B: int, L_act: int) -> int:
    return int(lib().hk_regen_workspace_bytes(ctypes.byref(shape), B, L_act))


def hk_regen_offsets(shape: hk_shape, B: int, L_act: int):
    """hk_regen_offsets: byte offsets of the regenerated K and V inside the workspace of hk_hybrid_decode_attn."""
    k, v = ctypes.c_size_t(), ctypes.c_size_t()
    st = lib().hk_regen_offsets(ctypes.byref(shape), B, L_act, ctypes.byref(k), ctypes.byref(v))
    if st != HK_OK:
        raise HybridKVError(st, "hk_regen_offsets")
    return int(k.value), int(v.value)


# ----------------------------------------------------------------------------- torch-facing calls
def _dev_ptr(t, name, dtype=None):
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a GPU tensor (there is no CPU path)" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s" % (name, dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _params(ln_w, ln_b, Wkv, bkv, prepared=None, el=None):
    import torch
    f16 = el or torch.float16
    pp = _dev_ptr(prepared, "prepared")
    return hk_layer_params(_dev_ptr(ln_w, "ln_w", f16).value, _dev_ptr(ln_b, "ln_b", f16).value,
                           _dev_ptr(Wkv, "Wkv", f16).value, _dev_ptr(bkv, "bkv", f16).value,
                           pp.value if pp is not None else None)


def hk_prepared_bytes(shape: hk_shape) -> int:
    return int(lib().hk_prepared_bytes(ctypes.byref(shape)))


def prepare_layer(ln_w, ln_b, Wkv, bkv, n_heads, stream=None):
    """hk_prepare_layer: returns the prepared-layer buffer (a uint8 GPU tensor) to pass as the fifth
    element of ``layer_params`` / the ``prepared`` argument."""
    d = ln_w.shape[0]
    shape = make_shape(d, n_heads, dtype=_dtype_code(Wkv))
    buf = new_workspace(hk_prepared_bytes(shape), ln_w.device)
    lp = _params(ln_w, ln_b, Wkv, bkv, el=Wkv.dtype)
    st = lib().hk_prepare_layer(ctypes.byref(shape), ctypes.byref(lp), _dev_ptr(buf, "prepared"), buf.numel(),
                                _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_prepare_layer")
    return buf


def new_workspace(nbytes: int, device="cuda"):
    """A device buffer for the ``workspace`` argument (torch's allocator aligns to >= 256 B)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def regen_kv(act, ln_w, ln_b, Wkv, bkv, n_heads, K_out=None, V_out=None, tok_off=0,
             ln_eps=1e-5, gemm_tile=0, workspace=None, stream=None, prepared=None):
    """hk_regen_kv: ``act[B, L_act, d]`` fp16 -> ``(K, V)``, each ``[B, H, L_cap, dh]`` fp16, rows
    ``tok_off .. tok_off+L_act`` written.  Allocates the outputs (L_cap = L_act) and the
    workspace when they are not given."""
    import torch
    B, L_act, d = act.shape
    el = act.dtype                                           # fp16, or bf16 (every tensor then)
    shape = make_shape(d, n_heads, ln_eps, gemm_tile=gemm_tile, dtype=_dtype_code(act))
    dh = d // n_heads
    if K_out is None:
        K_out = torch.empty((B, n_heads, L_act, dh), dtype=el, device=act.device)
        V_out = torch.empty_like(K_out)
    L_cap = K_out.shape[2]
    if workspace is None:
        workspace = new_workspace(hk_regen_workspace_bytes(shape, B, L_act), act.device)
    lp = _params(ln_w, ln_b, Wkv, bkv, prepared, el=el)
    st = lib().hk_regen_kv(ctypes.byref(shape), _dev_ptr(act, "act", el), B, L_act,
                           ctypes.byref(lp), _dev_ptr(K_out, "K_out", el),
                           _dev_ptr(V_out, "V_out", el), L_cap, tok_off,
                           _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_regen_kv")
    return K_out, V_out


def hybrid_decode_attn(q, K_cache, V_cache, act, layer_params, ratio, out=None, ln_eps=1e-5,
                       softmax_scale=0.0, attn_splits=0, gemm_tile=0, workspace=None, stream=None,
                       return_regen=False, events=None):
    """hk_hybrid_decode_attn: ``q[B,H,dh]``, ``K_cache,V_cache[B,H,L_kv,dh]`` (or None), ``act[B,L_act,d]``
    (or None), ``layer_params = (ln_w, ln_b, Wkv, bkv[, prepared])`` -> ``out[B,H,dh]`` (all fp16 GPU tensors).
    With ``return_regen`` also returns views of the regenerated K, V ``[B,H,L_act,dh]`` that
    the call left at the head of the workspace.  ``events`` (a ``hipevents.EventSet`` of 5)
    selects hk_hybrid_decode_attn_marked, which time-stamps the kernels of the step."""
    import torch
    B, H, dh = q.shape
    d = H * dh
    L_kv = 0 if K_cache is None else K_cache.shape[2]
    L_act = 0 if act is None else act.shape[1]
    f16 = q.dtype                                            # fp16, or bf16 (every tensor then)
    shape = make_shape(d, H, ln_eps, softmax_scale, attn_splits, gemm_tile, dtype=_dtype_code(q))
    if out is None:
        out = torch.empty((B, H, dh), dtype=f16, device=q.device)
    if workspace is None:
        workspace = new_workspace(hk_workspace_bytes(shape, B, L_kv, L_act), q.device)
    lp = _params(*layer_params[:4], prepared=layer_params[4] if len(layer_params) > 4 else None, el=f16)
    args = [ctypes.byref(shape), _dev_ptr(q, "q", f16),
            _dev_ptr(K_cache, "K_cache", f16), _dev_ptr(V_cache, "V_cache", f16), L_kv,
            _dev_ptr(act, "act", f16), L_act, B, ctypes.byref(lp), float(ratio),
            _dev_ptr(out, "out", f16), _dev_ptr(workspace, "workspace"),
            workspace.numel(), _stream_ptr(stream)]
    if events is None:
        st = lib().hk_hybrid_decode_attn(*args)
    else:
        st = lib().hk_hybrid_decode_attn_marked(*args, events.array, events.n)
    if st != HK_OK:
        raise HybridKVError(st, "hk_hybrid_decode_attn")
    if return_regen:
        n = B * H * L_act * dh
        k_off, v_off = hk_regen_offsets(shape, B, L_act)
        K = workspace[k_off:k_off + 2 * n].view(f16).view(B, H, L_act, dh)
        V = workspace[v_off:v_off + 2 * n].view(f16).view(B, H, L_act, dh)
        return out, K, V
    return out


def hybrid_decode_attn_static(q, K_cache, V_cache, act, layer_params, ratio, out, ln_eps=1e-5, softmax_scale=0.0,
                              attn_splits=0, gemm_tile=0, stream=None):
    """hk_hybrid_decode_attn_static: the step of ``hybrid_decode_attn`` on the library's static scratch array
    (no workspace, nothing allocated: ``out`` must be given)."""
    B, H, dh = q.shape
    L_kv = 0 if K_cache is None else K_cache.shape[2]
    L_act = 0 if act is None else act.shape[1]
    f16 = q.dtype
    shape = make_shape(H * dh, H, ln_eps, softmax_scale, attn_splits, gemm_tile, dtype=_dtype_code(q))
    lp = _params(*layer_params[:4], prepared=layer_params[4] if len(layer_params) > 4 else None, el=f16)
    st = lib().hk_hybrid_decode_attn_static(ctypes.byref(shape), _dev_ptr(q, "q", f16), _dev_ptr(K_cache, "K_cache", f16),
                                            _dev_ptr(V_cache, "V_cache", f16), L_kv, _dev_ptr(act, "act", f16), L_act, B,
                                            ctypes.byref(lp), float(ratio), _dev_ptr(out, "out", f16), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_hybrid_decode_attn_static")
    return out


def hk_two_stream_workspace_bytes(shape: hk_shape, B: int, L_kv: int, L_act: int) -> int:
    return int(lib().hk_two_stream_workspace_bytes(ctypes.byref(shape), B, L_kv, L_act))


def hybrid_decode_attn_two_stream(q, K_cache, V_cache, act, layer_params, ratio, side_stream, events, out=None, gemm_cus=0,
                                  ln_eps=1e-5, softmax_scale=0.0, workspace=None, stream=None, gemm_tile=0):
    """hk_hybrid_decode_attn_two_stream: the step with the attention over the cached segment on ``side_stream``
    (a torch stream; None = the same stream) beside the regeneration on ``stream``.  ``events``: a
    ``hipevents.EventSet`` of at least 2 (fork, join)."""
    import torch
    B, H, dh = q.shape
    L_kv = 0 if K_cache is None else K_cache.shape[2]
    L_act = 0 if act is None else act.shape[1]
    f16 = q.dtype
    shape = make_shape(H * dh, H, ln_eps, softmax_scale, 0, gemm_tile, dtype=_dtype_code(q))
    if out is None:
        out = torch.empty((B, H, dh), dtype=f16, device=q.device)
    if workspace is None:
        workspace = new_workspace(hk_two_stream_workspace_bytes(shape, B, L_kv, L_act), q.device)
    lp = _params(*layer_params[:4], prepared=layer_params[4] if len(layer_params) > 4 else None, el=f16)
    main = _stream_ptr(stream)
    side = main if side_stream is None else _stream_ptr(side_stream)
    st = lib().hk_hybrid_decode_attn_two_stream(
        ctypes.byref(shape), _dev_ptr(q, "q", f16), _dev_ptr(K_cache, "K_cache", f16), _dev_ptr(V_cache, "V_cache", f16), L_kv,
        _dev_ptr(act, "act", f16), L_act, B, ctypes.byref(lp), float(ratio), _dev_ptr(out, "out", f16),
        _dev_ptr(workspace, "workspace"), workspace.numel(), main, side, events.array[0], events.array[1], int(gemm_cus))
    if st != HK_OK:
        raise HybridKVError(st, "hk_hybrid_decode_attn_two_stream")
    return out


def hk_absorbed_workspace_bytes(shape: hk_shape, B: int, L_kv: int, L_act: int) -> int:
    return int(lib().hk_absorbed_workspace_bytes(ctypes.byref(shape), B, L_kv, L_act))


def hybrid_decode_attn_absorbed(q, K_cache, V_cache, act, layer_params, ratio, out=None, ln_eps=1e-5,
                                softmax_scale=0.0, attn_splits=0, workspace=None, stream=None):
    """hk_hybrid_decode_attn_absorbed: the arguments and the result of ``hybrid_decode_attn``, computed
    without regenerating K/V."""
    import torch
    B, H, dh = q.shape
    d = H * dh
    L_kv = 0 if K_cache is None else K_cache.shape[2]
    L_act = 0 if act is None else act.shape[1]
    f16 = q.dtype if q.dtype == torch.bfloat16 else torch.float16   # fp16, or bf16 (every tensor then)
    shape = make_shape(d, H, ln_eps, softmax_scale, attn_splits, 0, dtype=_dtype_code(q))
    if out is None:
        out = torch.empty((B, H, dh), dtype=f16, device=q.device)
    if workspace is None:
        workspace = new_workspace(hk_absorbed_workspace_bytes(shape, B, L_kv, L_act), q.device)
    lp = _params(*layer_params, el=f16)
    st = lib().hk_hybrid_decode_attn_absorbed(
        ctypes.byref(shape), _dev_ptr(q, "q", f16),
        _dev_ptr(K_cache, "K_cache", f16), _dev_ptr(V_cache, "V_cache", f16), L_kv,
        _dev_ptr(act, "act", f16), L_act, B, ctypes.byref(lp), float(ratio),
        _dev_ptr(out, "out", f16), _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_hybrid_decode_attn_absorbed")
    return out


def hk_qkv_workspace_bytes(shape: hk_shape, B: int) -> int:
    return int(lib().hk_qkv_workspace_bytes(ctypes.byref(shape), B))


def qkv_current(x_cur, ln_w, ln_b, Wkv, bkv, Wq, bq, n_heads, q_out=None, K_dst=None, V_dst=None, tok_pos=0,
                act_dst=None, act_pos=0, ln_eps=1e-5, workspace=None, stream=None):
    """hk_qkv_current: ``x_cur[B, d]`` (fp16, or bf16 with every other tensor) -> ``q[B, H, dh]``; writes the
    token's K/V row ``tok_pos`` into ``K_dst, V_dst[B, H, L_cap, dh]`` and/or its input row ``act_pos`` into
    ``act_dst[B, act_cap, d]`` when given."""
    import torch
    f16 = x_cur.dtype if x_cur.dtype == torch.bfloat16 else torch.float16
    B, d = x_cur.shape
    shape = make_shape(d, n_heads, ln_eps, dtype=_dtype_code(x_cur))
    dh = d // n_heads
    if q_out is None:
        q_out = torch.empty((B, n_heads, dh), dtype=f16, device=x_cur.device)
    if workspace is None:
        workspace = new_workspace(hk_qkv_workspace_bytes(shape, B), x_cur.device)
    lp = _params(ln_w, ln_b, Wkv, bkv, el=f16)
    L_cap = 0 if K_dst is None else K_dst.shape[2]
    act_cap = 0 if act_dst is None else act_dst.shape[1]
    st = lib().hk_qkv_current(ctypes.byref(shape), _dev_ptr(x_cur, "x_cur", f16), B, ctypes.byref(lp),
                              _dev_ptr(Wq, "Wq", f16), _dev_ptr(bq, "bq", f16), _dev_ptr(q_out, "q_out", f16),
                              _dev_ptr(K_dst, "K_dst", f16), _dev_ptr(V_dst, "V_dst", f16), L_cap, tok_pos,
                              _dev_ptr(act_dst, "act_dst", f16), act_cap, act_pos,
                              _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_qkv_current")
    return q_out


def qkv_current_paged(x_cur, ln_w, ln_b, Wkv, bkv, Wq, bq, n_heads, K_pool, V_pool, act_pool, block_table, seq_len,
                      block_tokens, q_out=None, ln_eps=1e-5, workspace=None, stream=None, store_mask=None):
    """hk_qkv_current_paged: ``x_cur[B, d]`` -> ``q[B, H, dh]``; the token of request r (token ``seq_len[r] - 1``)
    is written into the block its table entry names: K/V rows into ``K_pool, V_pool``, or the layer input into
    ``act_pool`` (pools may be None when empty; they are modified in place).  ``store_mask[B]`` int32 or None: zero =
    nothing is stored for the request (pass the ``grew`` array of ``paged_append``)."""
    import torch
    f16 = x_cur.dtype if x_cur.dtype == torch.bfloat16 else torch.float16
    B, d = x_cur.shape
    shape = make_shape(d, n_heads, ln_eps, dtype=_dtype_code(x_cur))
    if q_out is None:
        q_out = torch.empty((B, n_heads, d // n_heads), dtype=f16, device=x_cur.device)
    if workspace is None:
        workspace = new_workspace(hk_qkv_workspace_bytes(shape, B), x_cur.device)
    lp = _params(ln_w, ln_b, Wkv, bkv, el=f16)
    cache = make_paged_cache(K_pool, V_pool, act_pool, block_table, seq_len, None, 0, block_tokens, el=f16)
    st = lib().hk_qkv_current_paged(ctypes.byref(shape), _dev_ptr(x_cur, "x_cur", f16), B, ctypes.byref(lp),
                                    _dev_ptr(Wq, "Wq", f16), _dev_ptr(bq, "bq", f16), _dev_ptr(q_out, "q_out", f16),
                                    ctypes.byref(cache), _dev_ptr(store_mask, "store_mask", torch.int32),
                                    _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_qkv_current_paged")
    return q_out


def paged_append(block_table, seq_len, cu_tokens, counters, P_kv, P_act, block_tokens, act_host, kv_host, active=None,
                 stream=None, grew=None):
    """hk_paged_append: one more token for every (active) request, in place on the device: ``block_table[B,
    max_blocks]`` int32, ``seq_len[B]`` int32, ``cu_tokens[B+1]`` int64, ``counters[4]`` int32 (KV blocks in use,
    ACT blocks in use, requests that could not grow, unused), ``active[B]`` int32 or None, ``grew[B]`` int32 or None
    (written: 1 where the request took its token)."""
    import torch
    B, max_blocks = block_table.shape
    st = lib().hk_paged_append(_dev_ptr(block_table, "block_table", torch.int32), _dev_ptr(seq_len, "seq_len", torch.int32),
                               _dev_ptr(cu_tokens, "cu_tokens", torch.int64), _dev_ptr(counters, "counters", torch.int32),
                               _dev_ptr(active, "active", torch.int32), _dev_ptr(grew, "grew", torch.int32), B, max_blocks, int(block_tokens), int(P_kv), int(P_act),
                               int(act_host), int(kv_host), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_paged_append")


# ----------------------------------------------------------------------------- host-only policy arithmetic (Sec. 4.3)
def fit_line(n, t):
    """hk_fit_line: least-squares (slope, offset, r2) of samples t[i] over n[i]."""
    import numpy as np
    n = np.ascontiguousarray(n, dtype=np.float64)
    t = np.ascontiguousarray(t, dtype=np.float64)
    line, r2 = hk_line(), ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    st = lib().hk_fit_line(n.ctypes.data_as(dp), t.ctypes.data_as(dp), len(n), ctypes.byref(line), ctypes.byref(r2))
    if st != HK_OK:
        raise HybridKVError(st, "hk_fit_line")
    return line.slope, line.offset, r2.value


def host_block_allocation(T_load_w, T_kv_gen, T_load_kv, n_act_gpu, M_host, S_weight, S_kv):
    """hk_host_block_allocation (Algorithm 1); lines are (slope, offset) pairs.  Returns a dict of the six counts."""
    p = hk_alloc_params(T_load_w, hk_line(*T_kv_gen), hk_line(*T_load_kv), n_act_gpu, M_host, S_weight, S_kv)
    r = hk_alloc_result()
    st = lib().hk_host_block_allocation(ctypes.byref(p), ctypes.byref(r))
    if st != HK_OK:
        raise HybridKVError(st, "hk_host_block_allocation")
    return {k: int(getattr(r, k)) for k, _ in hk_alloc_result._fields_}


def next_block_type(n_act, n_kv, act_host, kv_host):
    """hk_next_block_type (Eq. 11): "ACT" or "KV"."""
    st = lib().hk_next_block_type(n_act, n_kv, act_host, kv_host)
    if st < 0:
        raise HybridKVError(st, "hk_next_block_type")
    return "ACT" if st == HK_BLOCK_ACT else "KV"


def minibatch_balance(T_kv_gen, T_load_kv, n_act_mb, n_kv_mb):
    """hk_minibatch_balance (Eq. 12, 13): (balance, F_b)."""
    b, c = ctypes.c_double(), ctypes.c_double()
    st = lib().hk_minibatch_balance(ctypes.byref(hk_line(*T_kv_gen)), ctypes.byref(hk_line(*T_load_kv)),
                                    n_act_mb, n_kv_mb, ctypes.byref(b), ctypes.byref(c))
    if st != HK_OK:
        raise HybridKVError(st, "hk_minibatch_balance")
    return b.value, c.value


# ----------------------------------------------------------------------------- paged hybrid cache
def make_paged_cache(K_pool, V_pool, act_pool, block_table, seq_len, cu_tokens, total_tokens, block_tokens,
                     n_act_used=None, el=None) -> hk_paged_cache:
    """Fills an hk_paged_cache from GPU tensors (pools may be None when empty; ``el``: their element type,
    fp16 unless given)."""
    import torch
    f16 = el or torch.float16
    P_kv = 0 if K_pool is None else K_pool.shape[0]
    P_act = 0 if act_pool is None else act_pool.shape[0]
    ptr = lambda t, name, dt: (_dev_ptr(t, name, dt).value if t is not None else None)
    return hk_paged_cache(ptr(K_pool, "K_pool", f16), ptr(V_pool, "V_pool", f16), ptr(act_pool, "act_pool", f16),
                          ptr(block_table, "block_table", torch.int32), ptr(seq_len, "seq_len", torch.int32),
                          ptr(cu_tokens, "cu_tokens", torch.int64), int(total_tokens), P_kv, P_act,
                          P_act if n_act_used is None else int(n_act_used), int(block_tokens),
                          0 if block_table is None else block_table.shape[1])


def paged_decode_attn(q, K_pool, V_pool, act_pool, block_table, seq_len, block_tokens, layer_params,
                      n_act_used=None, out=None, ln_eps=1e-5, softmax_scale=0.0, workspace=None, stream=None,
                      absorbed=False, cu_tokens=None, total_tokens=None):
    """hk_paged_decode_attn: ``q[B,H,dh]``, pools, ``block_table[B,max_blocks]`` int32, ``seq_len[B]`` int32 (GPU
    tensors) -> ``out[B,H,dh]``.  ``cu_tokens[B+1]`` int64 (GPU) and ``total_tokens`` are the prefix sums of
    ``seq_len`` and ``total_tokens`` their last element or an upper bound of it; the caller keeps them (on the device
    hk_paged_append maintains the prefix sums).  ``absorbed`` selects hk_paged_decode_attn_absorbed (the same step without regenerating
    K/V)."""
    import torch
    B, H, dh = q.shape
    el = q.dtype if q.dtype == torch.bfloat16 else torch.float16
    shape = make_shape(H * dh, H, ln_eps, softmax_scale, dtype=_dtype_code(q))
    if cu_tokens is None or total_tokens is None:
        raise ValueError("cu_tokens (int64 GPU tensor of B + 1 prefix sums) and total_tokens are required")
    if cu_tokens.dtype != torch.int64 or cu_tokens.numel() != B + 1 or not cu_tokens.is_cuda:
        raise ValueError("cu_tokens: int64 GPU tensor of B + 1 elements")
    cu, total = cu_tokens, int(total_tokens)
    cache = make_paged_cache(K_pool, V_pool, act_pool, block_table, seq_len, cu, total, block_tokens, n_act_used, el=el)
    if out is None:
        out = torch.empty((B, H, dh), dtype=el, device=q.device)
    size_fn = lib().hk_paged_absorbed_workspace_bytes if absorbed else lib().hk_paged_workspace_bytes
    entry = lib().hk_paged_decode_attn_absorbed if absorbed else lib().hk_paged_decode_attn
    if workspace is None:
        workspace = new_workspace(int(size_fn(ctypes.byref(shape), B, ctypes.byref(cache))), q.device)
    lp = _params(*layer_params, el=el) if layer_params is not None else None
    st = entry(ctypes.byref(shape), _dev_ptr(q, "q", el), B, ctypes.byref(cache),
                                    ctypes.byref(lp) if lp is not None else None, _dev_ptr(out, "out", el),
                                    _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_ptr(stream))
    if st != HK_OK:
        raise HybridKVError(st, "hk_paged_decode_attn_absorbed" if absorbed else "hk_paged_decode_attn")
    return out
