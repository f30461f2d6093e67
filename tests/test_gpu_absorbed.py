"""GPU parity of the decode step that never regenerates K/V (hk_hybrid_decode_attn_absorbed): its output
against the CPU oracle of the step (Eq. 7, 3, 4 written out), on the same seeded fp16 inputs and to the
same tolerance as the regenerating entry point, which it must also agree with.
"""
import numpy as np
import pytest
import torch

from paper_2501_01792_amd import synth
from test_gpu_parity import SMALL, _cfg, _check, _gpu, _oracle_hybrid, _run_hybrid, hk  # noqa: F401

pytestmark = pytest.mark.gpu


def _run_absorbed(hk, cfg, batch, prepared=False, **kw):
    lp = tuple(_gpu(batch[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    if prepared:
        lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    Kc = _gpu(batch["K_cache"]) if cfg.L_kv else None
    Vc = _gpu(batch["V_cache"]) if cfg.L_kv else None
    act = _gpu(batch["act"]) if cfg.L_act else None
    out = hk.hybrid_decode_attn_absorbed(_gpu(batch["q"]), Kc, Vc, act, lp, cfg.ratio, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


# Beyond the shared small cases: more than 32 / 64 heads (2 and 3 row blocks of the score product), more
# than 32 sequences (row blocks of the two weight products), more than 128 sequences (two launches of
# them), checkpoint counts that are not multiples of 16 or 32, a column count that is 64 mod 128.
SHAPES = SMALL + [
    _cfg("heads40", 2560, 40, 3, 150, 0.2, 21),
    _cfg("heads72", 4608, 72, 2, 90, 0.1, 22),
    _cfg("batch45", 512, 4, 45, 61, 0.5, 23),
    _cfg("batch130", 256, 4, 130, 40, 0.25, 24),
    _cfg("long_act", 512, 8, 2, 1500, 0.01, 25),
    # 65536 checkpoint rows or more select the score kernel with 128-row workgroups; 1030 rows per sequence
    # leave a last workgroup with 6 rows (three of its wavefronts own none)
    _cfg("block_rows", 256, 4, 64, 1030, 0.0, 26),
    # layers of 5120 features or more take the output projection that cuts the reduction axis over workgroups
    # (a head per workgroup, partial sums, a join kernel): head_dim 128 and 64, 1 and 2 row blocks of sequences,
    # and more than 128 sequences (two launches, the second with 2 rows)
    _cfg("wide_dh128", 5120, 40, 3, 24, 0.25, 27),
    _cfg("wide_dh64", 5120, 80, 45, 10, 0.2, 28),
    _cfg("wide_batch130", 5120, 40, 130, 6, 0.5, 29),
]


@pytest.mark.parametrize("prepared", [False, True])
@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: c.name)
def test_absorbed_step_matches_oracle(hk, oracle, cfg, prepared):
    print("case", cfg, "prepared", prepared, flush=True)
    batch = synth.make_batch(cfg)
    out = _run_absorbed(hk, cfg, batch, prepared=prepared)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, batch)
    _check("out", out, ref_out)


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[2], SHAPES[-5]], ids=lambda c: c.name)
def test_absorbed_agrees_with_regenerating_path(hk, cfg):
    print("case", cfg, flush=True)
    batch = synth.make_batch(cfg)
    a = _run_absorbed(hk, cfg, batch)
    b, _, _ = _run_hybrid(hk, cfg, batch)
    _check("absorbed vs regenerated", a, b)


def test_absorbed_peaked_scores(hk, oracle):
    """One checkpoint row that dominates the softmax and one cached row that does: the join of the two
    segments has to carry maxima that differ by hundreds of units of the exponent."""
    cfg = _cfg("peaked", 512, 4, 2, 96, 0.5, 31)
    batch = synth.make_batch(cfg)
    batch["q"] = (batch["q"].astype(np.float32) * 6).astype(np.float16)
    batch["K_cache"][0, :, 5, :] = (batch["q"][0].astype(np.float32) * 0.5).astype(np.float16)
    batch["act"][1, 7] = (batch["act"][1, 7].astype(np.float32) * 4).astype(np.float16)
    out = _run_absorbed(hk, cfg, batch)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, batch)
    _check("out", out, ref_out)


@pytest.mark.parametrize("prepared", [False, True])
def test_absorbed_rows_with_large_mean(hk, oracle, prepared):
    """Checkpoint rows whose mean is up to 200 times their spread: the mean has to cancel exactly in the
    carried query and in the weighted row sum (both kept in fp16), as it does in a LayerNorm; and the row
    statistics come from a single pass."""
    cfg = _cfg("shifted", 1024, 8, 2, 130, 0.0, 21)
    batch = synth.make_batch(cfg)
    rng = np.random.default_rng(5)
    act = batch["act"].astype(np.float32) * rng.uniform(0.1, 6.0, size=(cfg.B, cfg.L, 1)) + rng.uniform(-20, 20, size=(cfg.B, cfg.L, 1))
    batch["act"] = act.astype(np.float16)
    out = _run_absorbed(hk, cfg, batch, prepared=prepared)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, batch)
    _check("out", out, ref_out)


@pytest.mark.parametrize("cfg", [_cfg("outliers_slab", 1024, 8, 2, 130, 0.0, 21), _cfg("outliers_block", 256, 4, 64, 1030, 0.0, 26)],
                         ids=lambda c: c.name)
def test_absorbed_rows_with_outlier_features(hk, oracle, cfg):
    """A few feature channels that are 60 to 200 times the others in every row, the first channel among them (the
    rows enter the score product minus their first element): both forms of the score kernel, and the regenerating
    step beside them."""
    batch = synth.make_batch(cfg)
    act = batch["act"].astype(np.float32)
    for c, mag in ((0, 200.0), (3, -60.0), (cfg.d - 7, 60.0)):
        act[..., c] += mag
    batch["act"] = act.astype(np.float16)
    ref_out, _, _ = _oracle_hybrid(oracle, cfg, batch)
    _check("absorbed", _run_absorbed(hk, cfg, batch), ref_out)
    _check("regenerating", _run_hybrid(hk, cfg, batch)[0], ref_out)


def test_absorbed_repeatable_and_workspace_reuse(hk, oracle):
    """Two different problems through one workspace, larger first: the second result must not depend on
    what the first left behind (the padded tail of the weight rows is rewritten every call)."""
    big, small = SHAPES[2], SHAPES[1]
    from paper_2501_01792_amd import binding
    sh = binding.make_shape(big.d, big.n_heads, 1e-5, 0.0, 0, 0)
    n = max(binding.hk_absorbed_workspace_bytes(sh, big.B, big.L_kv, big.L_act),
            binding.hk_absorbed_workspace_bytes(binding.make_shape(small.d, small.n_heads, 1e-5, 0.0, 0, 0),
                                                small.B, small.L_kv, small.L_act))
    ws = binding.new_workspace(n, "cuda")
    ws.fill_(0x7f)
    for cfg in (big, small, small):
        batch = synth.make_batch(cfg)
        out = _run_absorbed(hk, cfg, batch, workspace=ws)
        ref_out, _, _ = _oracle_hybrid(oracle, cfg, batch)
        _check(cfg.name, out, ref_out)


def _sampled_pairs_check(hk, oracle, cfg, n_pairs=3, seed=5):
    batch = synth.make_batch(cfg, threads=16)
    print("  inputs drawn", flush=True)
    out = _run_absorbed(hk, cfg, batch, prepared=True)
    print("  GPU step done", flush=True)
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d
    rng = np.random.default_rng(seed)
    pairs = [(int(rng.integers(cfg.B)), int(rng.integers(H))) for _ in range(n_pairs)] + [(0, 0), (cfg.B - 1, H - 1)]
    got, ref = [], []
    for b, h in pairs:
        Kb = batch["K_cache"][b, h].astype(np.float64)
        Vb = batch["V_cache"][b, h].astype(np.float64)
        if cfg.L_act:
            xh = oracle.layernorm(batch["act"][b], batch["ln_w"], batch["ln_b"])
            sel = np.r_[h * dh:(h + 1) * dh, d + h * dh:d + (h + 1) * dh]
            kv = oracle.kv_projection(xh, batch["Wkv"][sel], batch["bkv"][sel])
            Kb = np.concatenate([Kb, kv[:, :dh]], axis=0)
            Vb = np.concatenate([Vb, kv[:, dh:]], axis=0)
        ref.append(oracle.decode_attention(batch["q"][b:b + 1, h:h + 1], Kb[None, None], Vb[None, None])[0, 0])
        got.append(out[b, h])
    _check("out[sampled (b,h)]", np.stack(got), np.stack(ref))


BIG = {
    "opt6.7b": synth.CONFIGS["opt6.7b"],
    "opt13b": synth.CONFIGS["opt13b"],
    "opt30b": synth.CONFIGS["opt30b"],                     # 131072 checkpoint rows: 128-row workgroups, 56 heads
    "opt66b": synth.CONFIGS["opt66b"],                     # 262144 checkpoint rows, d = 9216, 72 heads (3 head blocks)
    "opt66b@r0.5": synth.CONFIGS["opt66b"].with_ratio(0.5),   # the same layer with half of the context cached: the join
    "block_heads72": _cfg("block_heads72", 4608, 72, 17, 4000, 0.02, 27),   # the same kernel with 3 head blocks, ragged
    "dh64_big": _cfg("dh64_big", 2048, 32, 16, 2048, 0.5, 31),
    "one_long_sequence": _cfg("one_long_sequence", 1024, 8, 1, 40000, 0.1, 32),   # 36000 checkpoint rows of one sequence
}


@pytest.mark.parametrize("name", list(BIG))
def test_absorbed_full_size_sampled(hk, oracle, name):
    cfg = BIG[name]
    print("case", cfg, flush=True)
    torch.cuda.empty_cache()
    _sampled_pairs_check(hk, oracle, cfg)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("prepared", [False, True])
def test_absorbed_step_replays_from_a_hip_graph(hk, prepared):
    """The entry point allocates nothing and never synchronises: captured into a HIP graph and replayed on
    changing inputs, with eager work and synchronisations in between, it reproduces the eager result bit
    for bit (also when the layer is prepared inside the call)."""
    cfg = _cfg("graph", 1024, 8, 4, 320, 0.25, 26)
    batch = synth.make_batch(cfg)
    g = {k: _gpu(v) for k, v in batch.items()}
    lp = tuple(g[k] for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    if prepared:
        lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    shape = hk.make_shape(cfg.d, cfg.n_heads)
    n = hk.hk_absorbed_workspace_bytes(shape, cfg.B, cfg.L_kv, cfg.L_act)
    ws, ws_eager = hk.new_workspace(n), hk.new_workspace(n)
    out = torch.empty((cfg.B, cfg.n_heads, cfg.head_dim), dtype=torch.float16, device="cuda")
    q, act = g["q"].clone(), g["act"].clone()
    side = torch.cuda.Stream()                               # warm up first: kernel attributes are set on first use
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        hk.hybrid_decode_attn_absorbed(q, g["K_cache"], g["V_cache"], act, lp, cfg.ratio, out=out, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        hk.hybrid_decode_attn_absorbed(q, g["K_cache"], g["V_cache"], act, lp, cfg.ratio, out=out, workspace=ws,
                                       stream=torch.cuda.current_stream())
    rng = np.random.default_rng(6)
    for it in range(4):
        q.copy_(_gpu((rng.standard_normal(q.shape) * 2).astype(np.float16)))
        act.copy_(_gpu(rng.standard_normal(act.shape).astype(np.float16)))
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        ref = hk.hybrid_decode_attn_absorbed(q, g["K_cache"], g["V_cache"], act, lp, cfg.ratio, workspace=ws_eager)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), "replay %d differs from the eager step" % it
