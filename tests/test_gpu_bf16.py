"""GPU parity of the bfloat16 path (hk_prepare_layer, hk_regen_kv, hk_hybrid_decode_attn, hk_qkv_current,
hk_paged_decode_attn and the two entry points without regeneration, with HK_DTYPE_BF16)
against the CPU oracle fed with the same bf16-rounded inputs.

The benchmark's tolerance is stated for fp16.  A bf16 value carries 8 significant bits, so the output
rounding alone is up to 2^-8 of the value (fp16: 2^-11), and the prepared weights gamma * W are rounded
to bf16 as well.  The bar here, derived from that: max abs error <= 2^-7 * max |reference| (twice the
half-ulp of the largest value, for output rounding plus the rounding noise of the weights), relative L2
error <= 5e-3 as for fp16 (expected ~3e-3: 2^-8 / sqrt 3 from each of the two roundings).
"""
import numpy as np
import pytest
import torch

from paper_2501_01792_amd import synth
from test_gpu_parity import SMALL, _oracle_hybrid, hk  # noqa: F401

pytestmark = pytest.mark.gpu

REL_L2 = 5e-3


def _bf16(x):
    """numpy array -> (bf16 GPU tensor, the same values as float64 on the host)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.cuda(), t.float().numpy().astype(np.float64)


def _check(name, got, ref):
    got = got.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name + ": non-finite values"
    max_abs = np.abs(got - ref).max() if got.size else 0.0
    bound = 2.0 ** -7 * max(np.abs(ref).max(), 1e-30) if got.size else 0.0
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30) if got.size else 0.0
    print("%s: max_abs=%.3e (bound %.3e) rel_l2=%.3e" % (name, max_abs, bound, rel), flush=True)
    assert max_abs <= bound, "%s: max abs error %.3e > %.3e" % (name, max_abs, bound)
    assert rel <= REL_L2, "%s: relative L2 error %.3e" % (name, rel)


def _inputs(cfg):
    batch = synth.make_batch(cfg)
    g, h = {}, {}
    for k, v in batch.items():
        g[k], h[k] = _bf16(v)
    return g, h


@pytest.mark.parametrize("prepared", [False, True])
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_bf16_hybrid_step_matches_oracle(hk, oracle, cfg, prepared):
    print("case", cfg, "prepared", prepared, flush=True)
    g, h = _inputs(cfg)
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    if prepared:
        lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    out, K, V = hk.hybrid_decode_attn(g["q"], g["K_cache"] if cfg.L_kv else None, g["V_cache"] if cfg.L_kv else None,
                                      g["act"] if cfg.L_act else None, lp, cfg.ratio, return_regen=True)
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16 and K.dtype == torch.bfloat16
    ref_out, ref_K, ref_V = _oracle_hybrid(oracle, cfg, h)
    if cfg.L_act:
        _check("K_regen", K, ref_K[:, :, cfg.L_kv:])
        _check("V_regen", V, ref_V[:, :, cfg.L_kv:])
    _check("out", out, ref_out)


def test_bf16_regen_into_cache_slot(hk, oracle):
    """hk_regen_kv in bf16 writes rows tok_off .. tok_off + L_act of a larger cache and nothing else."""
    cfg = SMALL[2]
    g, h = _inputs(cfg)
    B, H, dh, L_act = cfg.B, cfg.n_heads, cfg.head_dim, cfg.L_act
    L_cap, off = L_act + 7, 3
    K = torch.full((B, H, L_cap, dh), 5.0, dtype=torch.bfloat16, device="cuda")
    V = torch.full((B, H, L_cap, dh), -5.0, dtype=torch.bfloat16, device="cuda")
    hk.regen_kv(g["act"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], H, K_out=K, V_out=V, tok_off=off)
    torch.cuda.synchronize()
    xh = oracle.layernorm(h["act"].reshape(-1, cfg.d), h["ln_w"], h["ln_b"])
    kv = oracle.kv_projection(xh, h["Wkv"], h["bkv"]).reshape(B, L_act, 2, H, dh)
    _check("K rows", K[:, :, off:off + L_act], kv[:, :, 0].transpose(0, 2, 1, 3))
    _check("V rows", V[:, :, off:off + L_act], kv[:, :, 1].transpose(0, 2, 1, 3))
    keep = np.ones(L_cap, bool); keep[off:off + L_act] = False
    assert (K[:, :, keep].float() == 5.0).all() and (V[:, :, keep].float() == -5.0).all()


def test_bf16_full_size_opt6p7b_sampled(hk, oracle):
    """The benchmark's workload in bf16: sampled K/V rows and sampled (sequence, head) outputs."""
    cfg = synth.CONFIGS["opt6.7b"]
    g, h = _inputs(cfg)
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    out, K, V = hk.hybrid_decode_attn(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio, return_regen=True)
    torch.cuda.synchronize()
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d
    rng = np.random.default_rng(9)
    rows = [(int(rng.integers(cfg.B)), int(rng.integers(cfg.L_act))) for _ in range(32)] + [(0, 0), (cfg.B - 1, cfg.L_act - 1)]
    xh = oracle.layernorm(np.stack([h["act"][b, t] for b, t in rows]), h["ln_w"], h["ln_b"])
    kv = oracle.kv_projection(xh, h["Wkv"], h["bkv"])
    _check("K_regen[sampled rows]", torch.stack([K[b, :, t, :].reshape(d) for b, t in rows]), kv[:, :d])
    _check("V_regen[sampled rows]", torch.stack([V[b, :, t, :].reshape(d) for b, t in rows]), kv[:, d:])
    got, ref = [], []
    for b, hd in [(int(rng.integers(cfg.B)), int(rng.integers(H))) for _ in range(3)] + [(cfg.B - 1, H - 1)]:
        xh = oracle.layernorm(h["act"][b], h["ln_w"], h["ln_b"])
        sel = np.r_[hd * dh:(hd + 1) * dh, d + hd * dh:d + (hd + 1) * dh]
        kvh = oracle.kv_projection(xh, h["Wkv"][sel], h["bkv"][sel])
        Kb = np.concatenate([h["K_cache"][b, hd], kvh[:, :dh]], axis=0)
        Vb = np.concatenate([h["V_cache"][b, hd], kvh[:, dh:]], axis=0)
        ref.append(oracle.decode_attention(h["q"][b:b + 1, hd:hd + 1], Kb[None, None], Vb[None, None])[0, 0])
        got.append(out[b, hd])
    _check("out[sampled (b,h)]", torch.stack(got), np.stack(ref))


@pytest.mark.parametrize("cfg", [synth.LayerConfig("tiny", 768, 12, 4, 256, 0.5, 0),
                                 synth.LayerConfig("rows33", 1024, 8, 33, 8, 0.5, 42),
                                 synth.LayerConfig("rows130_dh64", 1280, 20, 130, 8, 0.5, 43),
                                 synth.CONFIGS["opt6.7b"]], ids=lambda c: c.name)
def test_bf16_qkv_current_matches_oracle(hk, oracle, cfg):
    """QKV generation of the current token in bf16: q, the K/V rows written into the caches, the checkpoint copy."""
    print("case", cfg, flush=True)
    p, c = synth.make_params(cfg), synth.make_current_token(cfg)
    g, h = {}, {}
    for k, v in {**p, **c}.items():
        g[k], h[k] = _bf16(v)
    B, H, dh, d = cfg.B, cfg.n_heads, cfg.head_dim, cfg.d
    L_cap, pos, act_cap, apos = 5, 3, 4, 1
    K = torch.full((B, H, L_cap, dh), 7.0, dtype=torch.bfloat16, device="cuda")
    V = torch.full((B, H, L_cap, dh), -7.0, dtype=torch.bfloat16, device="cuda")
    A = torch.full((B, act_cap, d), 3.0, dtype=torch.bfloat16, device="cuda")
    q = hk.qkv_current(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H,
                       K_dst=K, V_dst=V, tok_pos=pos, act_dst=A, act_pos=apos)
    torch.cuda.synchronize()
    assert q.dtype == torch.bfloat16
    rq, rk, rv = oracle.qkv_current(h["x_cur"], h["ln_w"], h["ln_b"], h["Wq"], h["bq"], h["Wkv"], h["bkv"], H)
    _check("q", q, rq)
    _check("k", K[:, :, pos], rk)
    _check("v", V[:, :, pos], rv)
    assert torch.equal(A[:, apos], g["x_cur"])                     # the checkpoint is the layer input, bit for bit
    keep = [i for i in range(L_cap) if i != pos]
    assert (K[:, :, keep] == 7.0).all() and (V[:, :, keep] == -7.0).all()
    assert (A[:, [i for i in range(act_cap) if i != apos]] == 3.0).all()
    q2 = hk.qkv_current(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)                                      # q does not depend on whether K/V are produced


@pytest.mark.parametrize("case", [("dh64_bt16", 768, 12, 6, 300, 16, 0.5, [300, 1, 16, 0, 97, 255]),
                                  ("dh128_bt32", 1024, 8, 5, 700, 32, 0.4, [700, 33, 512, 64, 699]),
                                  ("all_kv", 512, 4, 4, 200, 16, 0.0, [200, 17, 128, 1])], ids=lambda c: c[0])
def test_bf16_paged_decode_matches_oracle(hk, case):
    """hk_paged_decode_attn in bf16 (block-table attention over KV blocks and regenerated checkpoint blocks)
    against the paged oracle fed with the same bf16-rounded pools, parameters and queries."""
    from oracle import paged_oracle as pgo
    from test_paged import _context
    name, d, H, B, L, bt, frac, seq_len = case
    print("case", case, flush=True)
    cfg = synth.LayerConfig(name, d, H, B, L, 0.5, 56)
    p, batch = _context(cfg, 13)
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, frac, seed=14)
    g, h = {}, {}
    for k, v in {**p, "q": batch["q"], "K_pool": paged["K_pool"], "V_pool": paged["V_pool"], "act_pool": paged["act_pool"]}.items():
        g[k], h[k] = _bf16(v)
    tb = torch.from_numpy(paged["block_table"]).cuda()
    sl = torch.from_numpy(paged["seq_len"]).cuda()
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    cs = np.concatenate([[0], np.cumsum(np.asarray(seq_len, dtype=np.int64))]).astype(np.int64)
    cu = {"cu_tokens": torch.from_numpy(cs).cuda(), "total_tokens": int(cs[-1])}
    out = hk.paged_decode_attn(g["q"], g["K_pool"], g["V_pool"], g["act_pool"], tb, sl, bt, lp, n_act_used=paged["n_act_used"],
                               **cu)
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16
    ref = pgo.paged_decode_attn(h["q"], h["K_pool"], h["V_pool"], h["act_pool"], paged["block_table"], paged["seq_len"], bt,
                                h["ln_w"], h["ln_b"], h["Wkv"], h["bkv"], H)
    _check("out", out, ref)
    for b in range(B):
        if seq_len[b] == 0:
            assert (out[b] == 0).all()
    out2 = hk.paged_decode_attn(g["q"], g["K_pool"], g["V_pool"], g["act_pool"], tb, sl, bt, lp, n_act_used=paged["n_act_used"],
                                absorbed=True, **cu)                # the same step without regeneration
    torch.cuda.synchronize()
    assert out2.dtype == torch.bfloat16
    _check("out, without regeneration", out2, ref)
    for b in range(B):
        if seq_len[b] == 0:
            assert (out2[b] == 0).all()


# ---- the step without regeneration (hk_hybrid_decode_attn_absorbed) on bf16 tensors.  It converts what it loads to
# fp16 and computes as it does for fp16 tensors, so its error is that of the fp16 step plus the output rounding to
# bf16; the oracle sees the same bf16-rounded inputs.  Same bar as the regenerating bf16 step.

def _absorbed_shapes():
    from test_gpu_absorbed import SHAPES
    return SHAPES


def _run_absorbed_bf16(hk, cfg, g, prepared):
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    if prepared:
        lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    out = hk.hybrid_decode_attn_absorbed(g["q"], g["K_cache"] if cfg.L_kv else None, g["V_cache"] if cfg.L_kv else None,
                                         g["act"] if cfg.L_act else None, lp, cfg.ratio)
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16
    return out


@pytest.mark.parametrize("prepared", [False, True])
@pytest.mark.parametrize("cfg", _absorbed_shapes(), ids=lambda c: c.name)
def test_bf16_absorbed_step_matches_oracle(hk, oracle, cfg, prepared):
    print("case", cfg, "prepared", prepared, flush=True)
    g, h = _inputs(cfg)
    out = _run_absorbed_bf16(hk, cfg, g, prepared)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, h)
    _check("out", out, ref_out)


def test_bf16_absorbed_rows_with_large_mean(hk, oracle):
    """Checkpoint rows whose mean is up to 200 times their spread, stored in bf16 (the spread is then a few units of
    the last place of the stored values): the mean has to cancel as it does in a LayerNorm."""
    from test_gpu_parity import _cfg
    cfg = _cfg("shifted", 1024, 8, 2, 130, 0.0, 21)
    batch = synth.make_batch(cfg)
    rng = np.random.default_rng(5)
    batch["act"] = batch["act"].astype(np.float32) * rng.uniform(0.1, 6.0, size=(cfg.B, cfg.L, 1)) \
        + rng.uniform(-20, 20, size=(cfg.B, cfg.L, 1))
    g, h = {}, {}
    for k, v in batch.items():
        g[k], h[k] = _bf16(v)
    out = _run_absorbed_bf16(hk, cfg, g, prepared=True)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, h)
    _check("out", out, ref_out)


def test_bf16_absorbed_peaked_scores(hk, oracle):
    """One checkpoint row that dominates the softmax and one cached row that does, in bf16."""
    from test_gpu_parity import _cfg
    cfg = _cfg("peaked", 512, 4, 2, 96, 0.5, 31)
    batch = synth.make_batch(cfg)
    batch["q"] = batch["q"].astype(np.float32) * 6
    batch["K_cache"][0, :, 5, :] = (batch["q"][0] * 0.5).astype(np.float16)
    batch["act"][1, 7] = (batch["act"][1, 7].astype(np.float32) * 4).astype(np.float16)
    g, h = {}, {}
    for k, v in batch.items():
        g[k], h[k] = _bf16(v)
    out = _run_absorbed_bf16(hk, cfg, g, prepared=False)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, h)
    _check("out", out, ref_out)


def test_bf16_absorbed_full_size_opt6p7b_sampled(hk, oracle):
    """The opt6.7b layer in bf16 without regeneration: sampled (sequence, head) outputs against the oracle, and
    agreement with the regenerating bf16 step on the whole output."""
    cfg = synth.CONFIGS["opt6.7b"]
    g, h = _inputs(cfg)
    out = _run_absorbed_bf16(hk, cfg, g, prepared=True)
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d
    rng = np.random.default_rng(11)
    got, ref = [], []
    for b, hd in [(int(rng.integers(cfg.B)), int(rng.integers(H))) for _ in range(3)] + [(0, 0), (cfg.B - 1, H - 1)]:
        xh = oracle.layernorm(h["act"][b], h["ln_w"], h["ln_b"])
        sel = np.r_[hd * dh:(hd + 1) * dh, d + hd * dh:d + (hd + 1) * dh]
        kvh = oracle.kv_projection(xh, h["Wkv"][sel], h["bkv"][sel])
        Kb = np.concatenate([h["K_cache"][b, hd], kvh[:, :dh]], axis=0)
        Vb = np.concatenate([h["V_cache"][b, hd], kvh[:, dh:]], axis=0)
        ref.append(oracle.decode_attention(h["q"][b:b + 1, hd:hd + 1], Kb[None, None], Vb[None, None])[0, 0])
        got.append(out[b, hd])
    _check("out[sampled (b,h)]", torch.stack(got), np.stack(ref))
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    regen = hk.hybrid_decode_attn(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio)
    torch.cuda.synchronize()
    _check("without regeneration vs regenerating", out, regen.float().cpu().numpy().astype(np.float64))


# ---- the two other forms of the regenerating step on bf16 tensors: the same kernels behind another entry point, so
# each must reproduce hk_hybrid_decode_attn's bf16 result (bit for bit where the arithmetic is the same) and stay
# within the bf16 bar of the oracle.

def test_bf16_static_scratch_call_matches_the_workspace_call(hk, oracle):
    cfg = SMALL[2]
    g, h = _inputs(cfg)
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    ref_gpu = hk.hybrid_decode_attn(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio)
    out = torch.full_like(ref_gpu, 7.0)
    hk.hybrid_decode_attn_static(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio, out)
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16 and torch.equal(out, ref_gpu)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, h)
    _check("out", out, ref_out)


def test_bf16_two_stream_step_matches_oracle(hk, oracle):
    from paper_2501_01792_amd.hipevents import EventSet
    cfg = SMALL[2]
    g, h = _inputs(cfg)
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    ev = EventSet(2)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    one = hk.hybrid_decode_attn_two_stream(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio, None, ev)
    torch.cuda.synchronize()
    two = hk.hybrid_decode_attn_two_stream(g["q"], g["K_cache"], g["V_cache"], g["act"], lp, cfg.ratio, side, ev)
    torch.cuda.synchronize()
    side.synchronize()
    ev.destroy()
    assert two.dtype == torch.bfloat16 and torch.equal(one, two), "the side stream changed the result"
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, h)
    _check("out", two, ref_out)
