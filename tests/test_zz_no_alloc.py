"""hk_hybrid_decode_attn_static (the step on the library's static scratch array, for callers that cannot
allocate) against hk_hybrid_decode_attn, through the C ABI: the same kernels on a different scratch address, so the
results must be bit-identical; and both within the step's tolerance of the oracle.  Two calls in a row, the second
on a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import hybridkv_oracle as ho
from paper_2501_01792_amd import binding as hk
from paper_2501_01792_amd import synth

MAX_ABS, REL_L2 = 2e-2, 5e-3


def _run_both(cfg, prepared, gemm_tile=0):
    b = synth.make_batch(cfg)
    g = {k: torch.from_numpy(v).cuda() for k, v in b.items()}
    lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
    if prepared:
        lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    Kc, Vc = (g["K_cache"], g["V_cache"]) if cfg.L_kv else (None, None)
    act = g["act"] if cfg.L_act else None
    ref_gpu = hk.hybrid_decode_attn(g["q"], Kc, Vc, act, lp, cfg.ratio, gemm_tile=gemm_tile)
    out = torch.full_like(ref_gpu, 7.0)
    hk.hybrid_decode_attn_static(g["q"], Kc, Vc, act, lp, cfg.ratio, out, gemm_tile=gemm_tile)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_gpu), "static-scratch call differs from the workspace call on %s" % cfg.name
    ref, _, _ = ho.hybrid_decode_attn(b["q"], b["K_cache"] if cfg.L_kv else None, b["V_cache"] if cfg.L_kv else None,
                                      b["act"] if cfg.L_act else None, b["ln_w"], b["ln_b"], b["Wkv"], b["bkv"], cfg.n_heads)
    got = out.float().cpu().numpy().astype(np.float64)
    err, rel = np.abs(got - ref).max(), np.linalg.norm(got - ref) / np.linalg.norm(ref)
    print("%s: max_abs=%.3e rel_l2=%.3e" % (cfg.name, err, rel), flush=True)
    assert err <= MAX_ABS and rel <= REL_L2


@pytest.mark.gpu
def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    # first a problem that fills most of the array and runs the large-problem projection kernel on a prepared
    # layer brought by the caller (d = 1024, 6 x 1024 checkpoint rows, 256-tiles asked for); then smaller ones that
    # reuse the dirty array: the tiny benchmark layer (small-problem kernel, layer not prepared), then one with no
    # checkpoints at all
    big = synth.LayerConfig("static_big", 1024, 8, 6, 2048, 0.5, 71)
    shape = hk.make_shape(big.d, big.n_heads, gemm_tile=256)
    need = hk.hk_workspace_bytes(shape, big.B, big.L_kv, big.L_act) - hk.hk_prepared_bytes(shape)
    assert hk.HK_STATIC_SCRATCH_BYTES // 2 < need <= hk.HK_STATIC_SCRATCH_BYTES
    _run_both(big, prepared=True, gemm_tile=256)
    _run_both(synth.CONFIGS["tiny"], prepared=False)
    _run_both(synth.LayerConfig("static_all_kv", 768, 12, 3, 200, 1.0, 72), prepared=False)


def test_static_scratch_call_rejects_what_does_not_fit():
    """Host checks (no GPU): a problem beyond the array is refused with its own status before anything else
    happens; the other checks are those of the workspace call."""
    FAKE = 0x7F0000001000
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    lp_prep = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, FAKE)

    def call(shape, L_kv, L_act, B, lp=lp, ratio=0.5, q=FAKE):
        return hk.lib().hk_hybrid_decode_attn_static(ctypes.byref(shape), q, FAKE, FAKE, L_kv, FAKE, L_act, B,
                                                     ctypes.byref(lp), ratio, FAKE, None)

    s67 = hk.make_shape(4096, 32)
    assert call(s67, 512, 512, 32) == hk.HK_ERR_STATIC_LIMIT             # 268 MB of regenerated K/V
    assert call(s67, 512, 512, 32, lp=lp_prep) == hk.HK_ERR_STATIC_LIMIT
    assert "HK_STATIC_SCRATCH_BYTES" in hk.status_string(hk.HK_ERR_STATIC_LIMIT)
    small = hk.make_shape(768, 12)
    assert call(small, 128, 128, 4, ratio=0.25) == hk.HK_ERR_RATIO
    assert call(small, 128, 128, 4, q=None) == hk.HK_ERR_NULL
    assert call(hk.make_shape(768, 11), 128, 128, 4) == hk.HK_ERR_SHAPE
    assert call(small, 0, 0, 4) == hk.HK_ERR_SHAPE
    assert call(small, 128, 128, 0) == hk.HK_OK                          # an empty batch: nothing to do
