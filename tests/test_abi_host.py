"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
function include/hybridkv.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2501_01792_amd import binding as hk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000      # never dereferenced: every call below must fail validation first


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hybridkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hk_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"hk_regen_kv", "hk_hybrid_decode_attn", "hk_workspace_bytes",
            "hk_regen_workspace_bytes", "hk_status_string", "hk_prepare_layer", "hk_prepared_bytes",
            "hk_hybrid_decode_attn_marked"} <= set(names)
    L = hk.lib()
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_matches_header():
    assert ctypes.sizeof(hk.hk_shape) == 32
    assert ctypes.sizeof(hk.hk_layer_params) == 40


def test_status_strings():
    for code in range(0, -8, -1):
        assert hk.status_string(code).startswith("HK_")
    assert "unknown" in hk.status_string(-99)


def test_workspace_bytes():
    s = hk.make_shape(4096, 32)
    B, L_kv, L_act = 32, 512, 512
    w = hk.hk_workspace_bytes(s, B, L_kv, L_act)
    regen = 2 * B * L_act * 4096 * 2
    prep = hk.hk_prepared_bytes(s)                                  # room for a per-call prepared layer (large problems)
    assert regen + B * L_act * 8 + prep <= w < regen + prep + (64 << 20)
    small = hk.hk_workspace_bytes(s, 1, 0, 64)                      # a small problem takes the 128-tile kernel: no such room
    assert small < prep
    assert hk.hk_regen_workspace_bytes(s, B, L_act) >= B * L_act * 8
    assert hk.hk_workspace_bytes(hk.make_shape(4096, 31), B, L_kv, L_act) == 0     # invalid shape
    assert hk.hk_workspace_bytes(s, 4, 100, 0) > 0
    # more splits -> more partials
    s64 = hk.make_shape(4096, 32, attn_splits=64)
    assert hk.hk_workspace_bytes(s64, 1, 0, 16384) > hk.hk_workspace_bytes(hk.make_shape(4096, 32, attn_splits=1), 1, 0, 16384)


def _attn(shape, q=FAKE, Kc=FAKE, Vc=FAKE, L_kv=128, act=FAKE, L_act=128, B=4, lp=None, ratio=0.5,
          out=FAKE, ws=FAKE, ws_bytes=1 << 40):
    if lp is None:
        lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    return hk.lib().hk_hybrid_decode_attn(ctypes.byref(shape), q, Kc, Vc, L_kv, act, L_act, B,
                                          ctypes.byref(lp) if lp != 0 else None, ratio, out, ws, ws_bytes, None)


def test_hybrid_decode_attn_rejects_bad_arguments():
    ok = hk.make_shape(768, 12)
    assert _attn(hk.make_shape(768, 11)) == hk.HK_ERR_SHAPE                 # d != H*dh
    assert _attn(hk.make_shape(768, 24)) == hk.HK_ERR_SHAPE                 # head_dim 32 unsupported
    bad = hk.make_shape(768, 12); bad.dtype = 2
    assert _attn(bad) == hk.HK_ERR_DTYPE
    bf = hk.make_shape(768, 12, dtype=hk.HK_DTYPE_BF16)                      # bf16: taken by the step ...
    assert _attn(bf, ratio=0.25) == hk.HK_ERR_RATIO and _attn(bf, q=None) == hk.HK_ERR_NULL
    assert hk.hk_workspace_bytes(bf, 4, 128, 128) > 0 and hk.hk_prepared_bytes(bf) == hk.hk_prepared_bytes(hk.make_shape(768, 12))
    # ... and by the QKV generation of the current token (same checks as in fp16: here the misplaced token) ...
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    assert hk.hk_qkv_workspace_bytes(bf, 4) == hk.hk_qkv_workspace_bytes(ok, 4) > 0
    assert hk.lib().hk_qkv_current(ctypes.byref(bf), FAKE, 4, ctypes.byref(lp), FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8,
                                   None, 0, 0, FAKE, 1 << 40, None) == hk.HK_ERR_SHAPE
    # ... and by the entry points that do not regenerate K/V (same scratch: their intermediate vectors are fp16 either way)
    assert hk.lib().hk_hybrid_decode_attn_absorbed(ctypes.byref(bf), FAKE, FAKE, FAKE, 128, FAKE, 128, 4, ctypes.byref(lp), 0.25,
                                                   FAKE, FAKE, 1 << 40, None) == hk.HK_ERR_RATIO
    assert hk.lib().hk_hybrid_decode_attn_absorbed(ctypes.byref(bf), FAKE, FAKE, FAKE, 128, None, 128, 4, ctypes.byref(lp), 0.5,
                                                   FAKE, FAKE, 1 << 40, None) == hk.HK_ERR_NULL
    assert hk.hk_absorbed_workspace_bytes(bf, 4, 128, 128) == hk.hk_absorbed_workspace_bytes(ok, 4, 128, 128) > 0
    assert _attn(hk.make_shape(768, 12, attn_splits=65)) == hk.HK_ERR_SHAPE
    assert _attn(hk.make_shape(768, 12, gemm_tile=64)) == hk.HK_ERR_SHAPE
    assert _attn(ok, ratio=1.5) == hk.HK_ERR_RATIO
    assert _attn(ok, ratio=-0.1) == hk.HK_ERR_RATIO
    assert _attn(ok, ratio=float("nan")) == hk.HK_ERR_RATIO
    assert _attn(ok, ratio=0.25) == hk.HK_ERR_RATIO                         # 128 of 256 is not 0.25
    assert _attn(ok, L_kv=0, L_act=0, ratio=0.0) == hk.HK_ERR_SHAPE         # empty context
    assert _attn(ok, L_kv=-1) == hk.HK_ERR_SHAPE
    assert _attn(ok, q=None) == hk.HK_ERR_NULL
    assert _attn(ok, out=None) == hk.HK_ERR_NULL
    assert _attn(ok, Kc=None) == hk.HK_ERR_NULL
    assert _attn(ok, act=None) == hk.HK_ERR_NULL
    assert _attn(ok, ws=None) == hk.HK_ERR_NULL
    assert _attn(ok, lp=hk.hk_layer_params(FAKE, None, FAKE, FAKE, None)) == hk.HK_ERR_NULL
    assert _attn(ok, q=FAKE + 8) == hk.HK_ERR_ALIGN
    assert _attn(ok, Vc=FAKE + 2) == hk.HK_ERR_ALIGN
    assert _attn(ok, ws=FAKE + 16) == hk.HK_ERR_ALIGN
    assert _attn(ok, ws_bytes=1024) == hk.HK_ERR_WORKSPACE
    need = hk.hk_workspace_bytes(ok, 4, 128, 128)
    assert _attn(ok, ws_bytes=need - 1) == hk.HK_ERR_WORKSPACE
    assert hk.lib().hk_hybrid_decode_attn(None, FAKE, FAKE, FAKE, 1, FAKE, 1, 1, None, 0.5,
                                          FAKE, FAKE, 1 << 30, None) == hk.HK_ERR_NULL
    # B == 0 is a no-op that still validates shape and ratio first
    assert _attn(ok, B=0) == hk.HK_OK
    assert _attn(ok, B=0, ratio=0.9) == hk.HK_ERR_RATIO


def test_absorbed_rejects_bad_arguments():
    """The variant that does not regenerate K/V validates like the step it mirrors, plus its own limits."""
    def call(shape, q=FAKE, Kc=FAKE, Vc=FAKE, L_kv=128, act=FAKE, L_act=128, B=4, lp=None, ratio=0.5,
             out=FAKE, ws=FAKE, ws_bytes=1 << 40):
        if lp is None:
            lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
        return hk.lib().hk_hybrid_decode_attn_absorbed(ctypes.byref(shape), q, Kc, Vc, L_kv, act, L_act, B,
                                                       ctypes.byref(lp), ratio, out, ws, ws_bytes, None)
    ok = hk.make_shape(768, 12)
    assert call(hk.make_shape(768, 11)) == hk.HK_ERR_SHAPE
    assert call(hk.make_shape(129 * 64, 129)) == hk.HK_ERR_SHAPE           # more than 128 heads
    assert call(ok, B=65536) == hk.HK_ERR_SHAPE
    assert call(ok, ratio=0.25) == hk.HK_ERR_RATIO
    assert call(ok, L_kv=0, L_act=0, ratio=0.0) == hk.HK_ERR_SHAPE
    assert call(ok, q=None) == hk.HK_ERR_NULL
    assert call(ok, act=None) == hk.HK_ERR_NULL
    assert call(ok, Kc=None) == hk.HK_ERR_NULL
    assert call(ok, lp=hk.hk_layer_params(FAKE, FAKE, None, FAKE, None)) == hk.HK_ERR_NULL
    assert call(ok, out=FAKE + 4) == hk.HK_ERR_ALIGN
    assert call(ok, act=FAKE + 8) == hk.HK_ERR_ALIGN
    need = hk.hk_absorbed_workspace_bytes(ok, 4, 128, 128)
    assert need > 0 and call(ok, ws_bytes=need - 1) == hk.HK_ERR_WORKSPACE
    assert call(ok, B=0) == hk.HK_OK
    # the workspace holds no regenerated K/V: far below the regenerating step's for a long checkpoint segment
    big = hk.make_shape(4096, 32)
    assert hk.hk_absorbed_workspace_bytes(big, 32, 0, 4096) < hk.hk_workspace_bytes(big, 32, 0, 4096) // 4
    assert hk.hk_absorbed_workspace_bytes(hk.make_shape(129 * 64, 129), 1, 0, 16) == 0


def _regen(shape, act=FAKE, B=4, L_act=128, lp=None, K=FAKE, V=FAKE, L_cap=128, tok_off=0, ws=FAKE, ws_bytes=1 << 40):
    if lp is None:
        lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    return hk.lib().hk_regen_kv(ctypes.byref(shape), act, B, L_act, ctypes.byref(lp), K, V, L_cap, tok_off,
                                ws, ws_bytes, None)


def test_regen_kv_rejects_bad_arguments():
    ok = hk.make_shape(768, 12)
    assert _regen(hk.make_shape(770, 12)) == hk.HK_ERR_SHAPE
    assert _regen(ok, L_cap=100) == hk.HK_ERR_SHAPE                         # rows would not fit
    assert _regen(ok, tok_off=1) == hk.HK_ERR_SHAPE
    assert _regen(ok, tok_off=-1, L_cap=256) == hk.HK_ERR_SHAPE
    assert _regen(ok, act=None) == hk.HK_ERR_NULL
    assert _regen(ok, K=None) == hk.HK_ERR_NULL
    assert _regen(ok, V=FAKE + 4) == hk.HK_ERR_ALIGN
    assert _regen(ok, lp=hk.hk_layer_params(FAKE, FAKE, None, FAKE, None)) == hk.HK_ERR_NULL
    assert _regen(ok, lp=hk.hk_layer_params(FAKE, FAKE, FAKE + 6, FAKE, None)) == hk.HK_ERR_ALIGN
    assert _regen(ok, ws_bytes=16) == hk.HK_ERR_WORKSPACE
    assert _regen(ok, L_act=0, L_cap=0) == hk.HK_OK                         # nothing to do
    assert _regen(ok, B=0) == hk.HK_OK


def test_prepare_layer_rejects_bad_arguments():
    ok = hk.make_shape(768, 12)
    need = hk.hk_prepared_bytes(ok)
    assert need >= 2 * 768 * 768 * 2 + 2 * 2 * 768 * 4
    assert hk.hk_prepared_bytes(hk.make_shape(768, 11)) == 0
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    call = lambda shape, lp, buf, n: hk.lib().hk_prepare_layer(ctypes.byref(shape), ctypes.byref(lp), buf, n, None)
    assert call(hk.make_shape(768, 11), lp, FAKE, need) == hk.HK_ERR_SHAPE
    assert call(ok, hk.hk_layer_params(FAKE, FAKE, None, FAKE, None), FAKE, need) == hk.HK_ERR_NULL
    assert call(ok, lp, None, need) == hk.HK_ERR_NULL
    assert call(ok, lp, FAKE + 16, need) == hk.HK_ERR_ALIGN
    assert call(ok, lp, FAKE, need - 1) == hk.HK_ERR_WORKSPACE
    # a misaligned prepared buffer inside the layer parameters is caught by the consumers
    assert _regen(ok, lp=hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, FAKE + 16)) == hk.HK_ERR_ALIGN


def test_qkv_current_rejects_bad_arguments():
    """Every check of hk_qkv_current runs on the host before a launch: no GPU is touched here."""
    ok = hk.make_shape(768, 12)
    need = hk.hk_qkv_workspace_bytes(ok, 4)
    assert need > 0                                              # a token amount: the call keeps its intermediates on chip
    assert hk.hk_qkv_workspace_bytes(hk.make_shape(768, 11), 4) == 0
    assert hk.hk_qkv_workspace_bytes(ok, 1000) == hk.hk_qkv_workspace_bytes(ok, 128)      # rows go 128 at a time
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)

    def call(shape=ok, x=FAKE, B=4, lp=lp, Wq=FAKE, bq=FAKE, q=FAKE, K=FAKE, V=FAKE, L_cap=8, pos=3,
             A=FAKE, acap=8, apos=2, ws=FAKE, n=need):
        return hk.lib().hk_qkv_current(ctypes.byref(shape), x, B, ctypes.byref(lp), Wq, bq, q, K, V, L_cap, pos,
                                       A, acap, apos, ws, n, None)

    assert call(shape=hk.make_shape(768, 11)) == hk.HK_ERR_SHAPE
    assert call(B=-1) == hk.HK_ERR_SHAPE
    assert call(B=0, x=None) == hk.HK_OK                              # nothing to do
    assert call(V=None) == hk.HK_ERR_NULL                             # K and V go together
    assert call(pos=8) == hk.HK_ERR_SHAPE and call(pos=-1) == hk.HK_ERR_SHAPE
    assert call(apos=8) == hk.HK_ERR_SHAPE
    assert call(x=None) == hk.HK_ERR_NULL and call(Wq=None) == hk.HK_ERR_NULL and call(q=None) == hk.HK_ERR_NULL
    assert call(lp=hk.hk_layer_params(FAKE, None, FAKE, FAKE, None)) == hk.HK_ERR_NULL
    assert call(x=FAKE + 8) == hk.HK_ERR_ALIGN and call(K=FAKE + 8) == hk.HK_ERR_ALIGN
    assert call(A=FAKE + 2) == hk.HK_ERR_ALIGN and call(ws=FAKE + 16) == hk.HK_ERR_ALIGN
    assert call(n=need - 1) == hk.HK_ERR_WORKSPACE


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 4, 768, dtype=torch.float16)
    w = torch.zeros(768, dtype=torch.float16)
    with pytest.raises(TypeError):
        hk.regen_kv(x, w, w, torch.zeros(1536, 768, dtype=torch.float16), torch.zeros(1536, dtype=torch.float16), 12,
                    K_out=torch.zeros(1, 12, 4, 64, dtype=torch.float16), V_out=torch.zeros(1, 12, 4, 64, dtype=torch.float16),
                    workspace=torch.zeros(1024, dtype=torch.uint8))


def test_algorithmic_byte_and_flop_counts():
    """The roofline's per-unit figures: a cached token costs 4d bytes per layer in fp16 (K and V),
    a checkpoint half of that (Sec. 4.1: an ACT block is half a KV block), and regenerating a
    token costs 4 d^2 flops (Eq. 7: d x 2d multiply-adds).  The 4d-byte figure is pinned by the
    KV traffic the paper quotes for OPT-30B with 1024-token inputs (Sec. 3.1): 21 GB per token
    step at batch 16 and 168 GB at batch 128, i.e. B * 1024 tokens * 48 layers * 4d bytes, d = 7168."""
    import bench
    from paper_2501_01792_amd import synth
    cfg = synth.CONFIGS["opt30b"]
    flops, attn_bytes = bench.algorithmic_counts(cfg)
    per_token_layer = attn_bytes / (cfg.B * cfg.L)
    assert per_token_layer == 4 * cfg.d
    assert flops == 4.0 * cfg.M * cfg.d ** 2
    gib = 1024.0 ** 3
    assert round(16 * 1024 * 48 * per_token_layer / gib, 1) == 21.0
    assert round(128 * 1024 * 48 * per_token_layer / gib, 1) == 168.0
    # the checkpoint of a token is d fp16 values: half of its K/V
    assert cfg.d * 2 * 2 == per_token_layer
