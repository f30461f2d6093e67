"""hk_hybrid_decode_attn_two_stream (the attention over the cached segment on a side stream beside the
regeneration; Sec. 4.2.2's overlap of KV generation with independent work, inside one GPU): host checks without a
GPU, then on the GPU against the oracle, against the single-stream issue of the same kernels (bit for bit) and
against hk_hybrid_decode_attn."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import hybridkv_oracle as ho
from paper_2501_01792_amd import binding as hk
from paper_2501_01792_amd import synth
from paper_2501_01792_amd.hipevents import EventSet

MAX_ABS, REL_L2 = 2e-2, 5e-3


def test_two_stream_rejects_bad_arguments():
    FAKE = 0x7F0000001000
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)
    ok = hk.make_shape(768, 12)

    def call(shape=ok, q=FAKE, L_kv=128, L_act=128, B=4, ratio=0.5, fork=FAKE, join=FAKE, n=1 << 40, cus=0, ws=FAKE):
        return hk.lib().hk_hybrid_decode_attn_two_stream(ctypes.byref(shape), q, FAKE, FAKE, L_kv, FAKE, L_act, B, ctypes.byref(lp),
                                                         ratio, FAKE, ws, n, None, None, fork, join, cus)

    need = hk.hk_two_stream_workspace_bytes(ok, 4, 128, 128)
    assert need >= hk.hk_workspace_bytes(ok, 4, 128, 128) > 0
    assert call(fork=None) == hk.HK_ERR_NULL and call(join=None) == hk.HK_ERR_NULL and call(q=None) == hk.HK_ERR_NULL
    assert call(ratio=0.25) == hk.HK_ERR_RATIO and call(cus=-1) == hk.HK_ERR_SHAPE and call(n=need - 1) == hk.HK_ERR_WORKSPACE
    assert call(shape=hk.make_shape(768, 11)) == hk.HK_ERR_SHAPE and call(ws=FAKE + 16) == hk.HK_ERR_ALIGN
    assert call(B=0) == hk.HK_OK
    assert hk.hk_two_stream_workspace_bytes(hk.make_shape(768, 11), 4, 128, 128) == 0


CASES = [
    synth.CONFIGS["tiny"],
    synth.LayerConfig("ragged", 1024, 8, 3, 427, 127 / 427, 81),
    synth.LayerConfig("big_tiles", 1024, 8, 16, 2048, 0.5, 82),            # 16384 checkpoint rows: the persistent kernel
    synth.LayerConfig("dh64", 768, 12, 5, 300, 0.75, 83),
    synth.LayerConfig("all_kv", 512, 8, 3, 200, 1.0, 84),                  # one segment only: the single-stream step
    synth.LayerConfig("all_act", 512, 8, 3, 200, 0.0, 85),
]


@pytest.mark.gpu
@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_two_stream_step(cfg):
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    print("case", cfg, flush=True)
    b = synth.make_batch(cfg)
    g = {k: torch.from_numpy(v).cuda() for k, v in b.items()}
    lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
    lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    Kc, Vc = (g["K_cache"], g["V_cache"]) if cfg.L_kv else (None, None)
    act = g["act"] if cfg.L_act else None
    ev = EventSet(2)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    one = hk.hybrid_decode_attn_two_stream(g["q"], Kc, Vc, act, lp, cfg.ratio, None, ev)            # everything on one stream
    torch.cuda.synchronize()
    two = hk.hybrid_decode_attn_two_stream(g["q"], Kc, Vc, act, lp, cfg.ratio, side, ev)           # side stream
    carved = hk.hybrid_decode_attn_two_stream(g["q"], Kc, Vc, act, lp, cfg.ratio, side, ev, gemm_cus=200)
    plain = hk.hybrid_decode_attn(g["q"], Kc, Vc, act, lp, cfg.ratio)
    torch.cuda.synchronize()
    side.synchronize()
    ev.destroy()
    assert torch.equal(one, two), "the side stream changed the result"
    assert torch.equal(one, carved), "the compute-unit carve-out changed the result"
    ref, _, _ = ho.hybrid_decode_attn(b["q"], b["K_cache"] if cfg.L_kv else None, b["V_cache"] if cfg.L_kv else None,
                                      b["act"] if cfg.L_act else None, b["ln_w"], b["ln_b"], b["Wkv"], b["bkv"], cfg.n_heads)
    got = two.float().cpu().numpy().astype(np.float64)
    err, rel = np.abs(got - ref).max(), np.linalg.norm(got - ref) / np.linalg.norm(ref)
    print("vs oracle: max_abs=%.3e rel_l2=%.3e" % (err, rel), flush=True)
    assert err <= MAX_ABS and rel <= REL_L2
    diff = (two.float() - plain.float()).abs().max().item()
    print("vs the single-stream entry point: max_abs=%.3e" % diff, flush=True)
    assert diff <= 4e-3                                       # two extra roundings to fp16 before the join


@pytest.mark.gpu
@pytest.mark.parametrize("d,H", [(128, 2), (192, 3), (256, 4), (320, 5), (448, 7), (1024, 8)], ids=lambda v: str(v))
def test_projection_on_few_compute_units_walks_many_tiles(d, H):
    """The persistent projection kernel confined to 3 compute units: every workgroup then computes several tiles in a
    row, with the load cursor crossing from one tile to the next while the matrix cores are two k blocks behind.
    Layers of 2, 3, 4, 5, 7 and 16 k blocks (a tile's first k block is its last but one, the main loop is empty, has an
    odd and an even number of passes), a ragged last row tile and a half last column tile; the regenerated K and V
    rows are checked one by one."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("walk_d%d" % d, d, H, 3, 801, 100 / 801, 90 + H)     # 3 x 701 = 2103 checkpoint rows: 9 row tiles
    print("case", cfg, flush=True)
    b = synth.make_batch(cfg)
    g = {k: torch.from_numpy(v).cuda() for k, v in b.items()}
    lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
    shape = hk.make_shape(d, H, gemm_tile=256)
    ws = hk.new_workspace(hk.hk_two_stream_workspace_bytes(shape, cfg.B, cfg.L_kv, cfg.L_act), "cuda")
    ev = EventSet(2)
    out = hk.hybrid_decode_attn_two_stream(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio, None, ev, gemm_cus=3,
                                           workspace=ws, gemm_tile=256)
    torch.cuda.synchronize()
    n = cfg.B * H * cfg.L_act * cfg.head_dim
    k_off, v_off = hk.hk_regen_offsets(shape, cfg.B, cfg.L_act)
    K = ws[k_off:k_off + 2 * n].view(torch.float16).view(cfg.B, H, cfg.L_act, cfg.head_dim).float().cpu().numpy()
    V = ws[v_off:v_off + 2 * n].view(torch.float16).view(cfg.B, H, cfg.L_act, cfg.head_dim).float().cpu().numpy()
    ref_out, ref_K, ref_V = ho.hybrid_decode_attn(b["q"], b["K_cache"], b["V_cache"], b["act"], b["ln_w"], b["ln_b"], b["Wkv"],
                                                  b["bkv"], H)
    ev.destroy()
    for name, got, ref in (("K_regen", K, ref_K[:, :, cfg.L_kv:]), ("V_regen", V, ref_V[:, :, cfg.L_kv:]),
                           ("out", out.float().cpu().numpy(), ref_out)):
        err = np.abs(got - ref).max()
        rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
        print("%s: max_abs=%.3e rel_l2=%.3e" % (name, err, rel), flush=True)
        assert err <= MAX_ABS and rel <= REL_L2, (name, err, rel)
