"""GPU parity of the current-token QKV generation and write-back (hk_qkv_current) against the CPU
oracle, and of the decode step that includes the current token through either store.

Tolerances as for the rest of the path: max abs error <= 2e-2, relative L2 error <= 5e-3.
"""
import numpy as np
import pytest
import torch

from paper_2501_01792_amd import synth

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
REL_L2 = 5e-3


@pytest.fixture(scope="module")
def hk():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    from paper_2501_01792_amd import binding
    binding.lib()
    return binding


def _gpu(x):
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _check(name, got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name + ": non-finite values"
    max_abs = np.abs(got - ref).max()
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    print("%s: max_abs=%.3e rel_l2=%.3e" % (name, max_abs, rel), flush=True)
    assert max_abs <= MAX_ABS, "%s: max abs error %.3e" % (name, max_abs)
    assert rel <= REL_L2, "%s: relative L2 error %.3e" % (name, rel)


CASES = [
    synth.LayerConfig("tiny", 768, 12, 4, 256, 0.5, 0),
    synth.LayerConfig("one_row", 256, 4, 1, 8, 0.5, 41),
    synth.LayerConfig("rows33", 1024, 8, 33, 8, 0.5, 42),            # two row blocks, ragged
    synth.LayerConfig("rows130_dh64", 1280, 20, 130, 8, 0.5, 43),    # more rows than one launch takes; d/64 = 20 steps
    synth.CONFIGS["opt6.7b"],
    synth.CONFIGS["opt13b"],                                         # B = 64, d = 5120
    synth.CONFIGS["opt30b"],                                         # B = 128, d = 7168
    synth.CONFIGS["opt66b"],                                         # B = 64, d = 9216: the reduction axis in 2 parts
    synth.LayerConfig("rows96_d9216", 9216, 72, 96, 8, 0.5, 45),     # three row blocks at the widest layer
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_qkv_current_matches_oracle_and_writes_only_its_rows(hk, oracle, cfg):
    print("case", cfg, flush=True)
    p, c = synth.make_params(cfg), synth.make_current_token(cfg)
    B, H, dh, d = cfg.B, cfg.n_heads, cfg.head_dim, cfg.d
    L_cap, pos, act_cap, apos = 5, 3, 4, 1
    K = torch.full((B, H, L_cap, dh), 7.0, dtype=torch.float16, device="cuda")
    V = torch.full((B, H, L_cap, dh), -7.0, dtype=torch.float16, device="cuda")
    A = torch.full((B, act_cap, d), 3.0, dtype=torch.float16, device="cuda")
    g = {k: _gpu(v) for k, v in {**p, **c}.items()}
    q = hk.qkv_current(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H,
                       K_dst=K, V_dst=V, tok_pos=pos, act_dst=A, act_pos=apos)
    torch.cuda.synchronize()
    rq, rk, rv = oracle.qkv_current(c["x_cur"], p["ln_w"], p["ln_b"], c["Wq"], c["bq"], p["Wkv"], p["bkv"], H)
    K, V, A = K.cpu().numpy(), V.cpu().numpy(), A.cpu().numpy()
    _check("q", q.cpu().numpy(), rq)
    _check("k", K[:, :, pos], rk)
    _check("v", V[:, :, pos], rv)
    assert np.array_equal(A[:, apos], c["x_cur"])                    # the checkpoint is the layer input, bit for bit
    keep = np.ones(L_cap, bool); keep[pos] = False
    assert (K[:, :, keep] == 7.0).all() and (V[:, :, keep] == -7.0).all()
    akeep = np.ones(act_cap, bool); akeep[apos] = False
    assert (A[:, akeep] == 3.0).all()
    # q only: no K/V, no checkpoint
    q2 = hk.qkv_current(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)


@pytest.mark.parametrize("route", ["kv", "act"])
def test_decode_step_with_current_token(hk, oracle, route):
    """Sec. 4.2.2 end to end: QKV generation of the input token, the token joins one of the two
    stores, attention over cached ++ regenerated K/V including it."""
    cfg = synth.LayerConfig("step", 1024, 8, 6, 300, 100 / 300, 44)
    p, c, b = synth.make_params(cfg), synth.make_current_token(cfg), synth.make_batch(cfg)
    B, H, dh, d, L_kv, L_act = cfg.B, cfg.n_heads, cfg.head_dim, cfg.d, cfg.L_kv, cfg.L_act
    g = {k: _gpu(v) for k, v in {**p, **c}.items()}
    Kc = torch.zeros((B, H, L_kv + 1, dh), dtype=torch.float16, device="cuda")
    Vc = torch.zeros_like(Kc)
    Kc[:, :, :L_kv] = _gpu(b["K_cache"]); Vc[:, :, :L_kv] = _gpu(b["V_cache"])
    act = torch.zeros((B, L_act + 1, d), dtype=torch.float16, device="cuda")
    act[:, :L_act] = _gpu(b["act"])
    lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
    rq, rk, rv = oracle.qkv_current(c["x_cur"], p["ln_w"], p["ln_b"], c["Wq"], c["bq"], p["Wkv"], p["bkv"], H)
    if route == "kv":
        q = hk.qkv_current(g["x_cur"], *lp, g["Wq"], g["bq"], H, K_dst=Kc, V_dst=Vc, tok_pos=L_kv)
        out = hk.hybrid_decode_attn(q, Kc, Vc, act[:, :L_act].contiguous(), lp, (L_kv + 1) / (cfg.L + 1))
        ref, _, _ = oracle.hybrid_decode_attn(rq, np.concatenate([b["K_cache"].astype(np.float64), rk[:, :, None]], axis=2),
                                              np.concatenate([b["V_cache"].astype(np.float64), rv[:, :, None]], axis=2),
                                              b["act"], p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
    else:
        q = hk.qkv_current(g["x_cur"], *lp, g["Wq"], g["bq"], H, act_dst=act, act_pos=L_act)
        out = hk.hybrid_decode_attn(q, Kc[:, :, :L_kv].contiguous(), Vc[:, :, :L_kv].contiguous(), act, lp, L_kv / (cfg.L + 1))
        ref, _, _ = oracle.hybrid_decode_attn(rq, b["K_cache"], b["V_cache"],
                                              np.concatenate([b["act"], c["x_cur"][:, None]], axis=1),
                                              p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
    torch.cuda.synchronize()
    _check("out[%s]" % route, out.cpu().numpy(), ref)
