"""Paged hybrid cache (Sec. 4.1, 4.2.1): pins of the paged oracle (CPU), host-side argument checks of
hk_paged_decode_attn (CPU), and GPU parity against the oracle through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import hybridkv_oracle as ho
from oracle import paged_oracle as pgo
from paper_2501_01792_amd import binding as hk
from paper_2501_01792_amd import synth

MAX_ABS = 2e-2
REL_L2 = 5e-3


def _prefix_sums(seq_len):
    """cu_tokens (int64, on the GPU) and their total, from the request lengths the test holds on the host."""
    cu = np.concatenate([[0], np.cumsum(np.asarray(seq_len, dtype=np.int64))]).astype(np.int64)
    return {"cu_tokens": torch.from_numpy(cu).cuda(), "total_tokens": int(cu[-1])}


def _context(cfg, rng_seed):
    """Contiguous context of cfg.B requests of cfg.L tokens: layer inputs of every token and K/V rows (any
    numbers: a cache may hold anything) in fp16, plus layer parameters and queries."""
    rng = np.random.default_rng(rng_seed)
    B, H, dh, d, L = cfg.B, cfg.n_heads, cfg.head_dim, cfg.d, cfg.L
    p = synth.make_params(cfg)
    batch = {"act_full": rng.standard_normal((B, L, d)).astype(np.float16),
             "K_full": (rng.standard_normal((B, H, L, dh)) * 0.02 * np.sqrt(d)).astype(np.float16),
             "V_full": (rng.standard_normal((B, H, L, dh)) * 0.02 * np.sqrt(d)).astype(np.float16),
             "q": (rng.standard_normal((B, H, dh)) * 0.02 * np.sqrt(d)).astype(np.float16)}
    return p, batch


def _reference_by_regrouping(cfg, p, batch, paged, bt):
    """What the pinned contiguous oracle gives when each request's KV-block tokens are handed over as its
    cache and its ACT-block tokens as its checkpoints (attention does not depend on token order)."""
    out = np.zeros((cfg.B, cfg.n_heads, cfg.head_dim))
    for b in range(cfg.B):
        n = int(paged["seq_len"][b])
        if n == 0:
            continue
        tok_kv = [t for t in range(n) if not paged["kinds"][b][t // bt]]
        tok_act = [t for t in range(n) if paged["kinds"][b][t // bt]]
        Kc = batch["K_full"][b:b + 1][:, :, tok_kv] if tok_kv else None
        Vc = batch["V_full"][b:b + 1][:, :, tok_kv] if tok_kv else None
        act = batch["act_full"][b:b + 1][:, tok_act] if tok_act else None
        o, _, _ = ho.hybrid_decode_attn(batch["q"][b:b + 1], Kc, Vc, act, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], cfg.n_heads)
        out[b] = o[0]
    return out


# ------------------------------------------------------------------ oracle pins (CPU)
@pytest.mark.parametrize("bt,frac", [(16, 0.5), (32, 0.3), (16, 0.0), (16, 1.0), (64, 0.7)])
def test_paged_oracle_equals_contiguous_oracle(bt, frac):
    cfg = synth.LayerConfig("pg", 64, 4, 5, 150, 0.5, 51)
    p, batch = _context(cfg, 1)
    seq_len = [150, 1, 16, 0, 97]                     # full, single token, exactly one block, empty, ragged
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, frac, seed=2)
    got = pgo.paged_decode_attn(batch["q"], paged["K_pool"], paged["V_pool"], paged["act_pool"], paged["block_table"],
                                paged["seq_len"], bt, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], cfg.n_heads)
    ref = _reference_by_regrouping(cfg, p, batch, paged, bt)
    np.testing.assert_allclose(got, ref, atol=1e-12)
    assert (got[3] == 0).all()                        # the empty request


def test_paged_oracle_single_block_by_hand():
    """One request, one KV block holding two tokens with k = v = (1,-1), (-1,1), q chosen so that the weights
    are 3/4 and 1/4 (the hand-worked case of the contiguous oracle): out = (1/2, -1/2); rows of the block
    beyond the request's length must not matter."""
    bt = 16
    K = np.full((1, 1, bt, 2), 99.0); K[0, 0, 0] = (1, -1); K[0, 0, 1] = (-1, 1)
    q = np.array([[[np.log(3.0) / np.sqrt(2.0), 0.0]]])
    out = pgo.paged_decode_attn(q, K, K.copy(), np.zeros((0, bt, 2)), np.array([[0]], dtype=np.int32), [2], bt,
                                np.ones(2), np.zeros(2), np.zeros((4, 2)), np.zeros(4), 1, eps=0.0)
    np.testing.assert_allclose(out[0, 0], (0.5, -0.5), atol=1e-14)


# ------------------------------------------------------------------ host-side checks (CPU)
def test_paged_rejects_bad_arguments():
    FAKE = 0x10000
    ok = hk.make_shape(768, 12)
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)

    def cache(**kw):
        f = dict(K_pool=FAKE, V_pool=FAKE, act_pool=FAKE, block_table=FAKE, seq_len=FAKE, cu_tokens=FAKE,
                 total_tokens=100, P_kv=8, P_act=8, n_act_used=4, block_tokens=16, max_blocks=8)
        f.update(kw)
        return hk.hk_paged_cache(**f)

    def call(shape=ok, q=FAKE, B=2, c=None, lp=lp, out=FAKE, ws=FAKE, n=None):
        c = c or cache()
        need = hk.lib().hk_paged_workspace_bytes(ctypes.byref(shape), B, ctypes.byref(c))
        return hk.lib().hk_paged_decode_attn(ctypes.byref(shape), q, B, ctypes.byref(c), ctypes.byref(lp) if lp else None,
                                             out, ws, need if n is None else n, None)

    need = hk.lib().hk_paged_workspace_bytes(ctypes.byref(ok), 2, ctypes.byref(cache()))
    assert need >= 2 * 4 * 16 * 768 * 2                                  # the regenerated K and V of the ACT blocks in use
    assert call(c=cache(block_tokens=24)) == hk.HK_ERR_SHAPE            # not a power of two
    assert call(c=cache(block_tokens=8)) == hk.HK_ERR_SHAPE
    assert call(c=cache(n_act_used=9)) == hk.HK_ERR_SHAPE                # more than the pool holds
    assert call(c=cache(total_tokens=2 * 8 * 16 + 1)) == hk.HK_ERR_SHAPE  # more tokens than the tables can map
    assert call(c=cache(P_kv=0, n_act_used=0, K_pool=None, V_pool=None)) == hk.HK_ERR_SHAPE   # tokens but no blocks
    assert call(B=0, q=None, c=cache(total_tokens=0)) == hk.HK_OK
    assert call(q=None) == hk.HK_ERR_NULL and call(c=cache(block_table=None)) == hk.HK_ERR_NULL
    assert call(c=cache(K_pool=None)) == hk.HK_ERR_NULL and call(c=cache(act_pool=None)) == hk.HK_ERR_NULL
    assert call(lp=None) == hk.HK_ERR_NULL                               # ACT blocks in use need the layer
    assert call(c=cache(cu_tokens=FAKE + 4)) == hk.HK_ERR_ALIGN and call(q=FAKE + 2) == hk.HK_ERR_ALIGN
    assert call(n=need - 1) == hk.HK_ERR_WORKSPACE

    # the entry point that does not regenerate K/V: the same checks, its own limits and its own (smaller) workspace
    def call2(shape=ok, q=FAKE, B=2, c=None, lp=lp, out=FAKE, ws=FAKE, n=None):
        c = c or cache()
        need2 = hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(shape), B, ctypes.byref(c))
        return hk.lib().hk_paged_decode_attn_absorbed(ctypes.byref(shape), q, B, ctypes.byref(c), ctypes.byref(lp) if lp else None,
                                                      out, ws, need2 if n is None else n, None)

    need2 = hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(ok), 2, ctypes.byref(cache()))
    assert need2 > 0
    assert call2(c=cache(block_tokens=24)) == hk.HK_ERR_SHAPE and call2(c=cache(n_act_used=9)) == hk.HK_ERR_SHAPE
    assert call2(shape=hk.make_shape(129 * 64, 129)) == hk.HK_ERR_SHAPE       # more than 128 heads
    assert call2(q=None) == hk.HK_ERR_NULL and call2(c=cache(act_pool=None)) == hk.HK_ERR_NULL and call2(lp=None) == hk.HK_ERR_NULL
    assert call2(out=FAKE + 2) == hk.HK_ERR_ALIGN and call2(n=need2 - 1) == hk.HK_ERR_WORKSPACE
    assert call2(B=0, q=None, c=cache(total_tokens=0)) == hk.HK_OK
    big = hk.hk_paged_cache(K_pool=FAKE, V_pool=FAKE, act_pool=FAKE, block_table=FAKE, seq_len=FAKE, cu_tokens=FAKE,
                            total_tokens=32 * 4096, P_kv=8, P_act=32 * 256, n_act_used=32 * 256, block_tokens=16, max_blocks=256)
    s67 = hk.make_shape(4096, 32)
    assert hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(s67), 32, ctypes.byref(big)) < \
        hk.lib().hk_paged_workspace_bytes(ctypes.byref(s67), 32, ctypes.byref(big)) // 4
    # bfloat16: taken by both entry points, with the same checks
    bf = hk.make_shape(768, 12, dtype=hk.HK_DTYPE_BF16)
    assert call(shape=bf, q=None) == hk.HK_ERR_NULL and call(shape=bf, c=cache(block_tokens=24)) == hk.HK_ERR_SHAPE
    assert hk.lib().hk_paged_workspace_bytes(ctypes.byref(bf), 2, ctypes.byref(cache())) >= need     # always a prepared layer inside
    assert hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(bf), 2, ctypes.byref(cache())) == \
        hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(ok), 2, ctypes.byref(cache())) > 0
    assert hk.lib().hk_paged_decode_attn_absorbed(ctypes.byref(bf), None, 2, ctypes.byref(cache()), ctypes.byref(lp), FAKE, FAKE,
                                                  1 << 40, None) == hk.HK_ERR_NULL
    assert hk.lib().hk_paged_decode_attn_absorbed(ctypes.byref(bf), FAKE, 2, ctypes.byref(cache(block_tokens=24)), ctypes.byref(lp),
                                                  FAKE, FAKE, 1 << 40, None) == hk.HK_ERR_SHAPE


# ------------------------------------------------------------------ GPU parity
def _check(name, got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), name
    max_abs = np.abs(got - ref).max()
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    print("%s: max_abs=%.3e rel_l2=%.3e" % (name, max_abs, rel), flush=True)
    assert max_abs <= MAX_ABS and rel <= REL_L2, (name, max_abs, rel)


GPU_CASES = [
    # name, d, H, B, L, block_tokens, ACT share of the blocks, request lengths (None: random ragged)
    ("dh64_bt16", 768, 12, 6, 300, 16, 0.5, [300, 1, 16, 0, 97, 255]),
    ("dh128_bt32", 1024, 8, 5, 700, 32, 0.4, None),
    ("all_kv", 512, 4, 4, 200, 16, 0.0, None),
    ("all_act", 512, 4, 3, 130, 64, 1.0, None),
    # requests of one kind each beside mixed ones: the cached and the checkpoint part of a request can be empty
    ("one_kind_each", 512, 4, 6, 210, 16, [0.0, 1.0, 0.5, 1.0, 0.0, 0.9], [210, 209, 100, 16, 17, 0]),
    ("opt6.7b_shape", 4096, 32, 32, 1024, 16, 0.5, None),     # the benchmark layer with ragged requests
    # the largest layer of the benchmark contract (d = 9216, 72 heads) with ragged requests of up to 2048 tokens
    ("opt66b_shape", 9216, 72, 24, 2048, 16, 0.5, None),
]


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [False, True], ids=["regenerating", "absorbed"])
@pytest.mark.parametrize("case", GPU_CASES, ids=lambda c: c[0])
def test_paged_decode_matches_oracle(case, absorbed):
    name, d, H, B, L, bt, frac, lens = case
    print("case", case[:7], "absorbed", absorbed, flush=True)
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig(name, d, H, B, L, 0.5, 52)
    p, batch = _context(cfg, 3)
    rng = np.random.default_rng(4)
    seq_len = lens if lens is not None else [int(v) for v in rng.integers(1, L + 1, B)]
    if lens is None:
        seq_len[0] = L
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, frac, seed=5)
    g = lambda x: None if x is None or x.shape[0] == 0 else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    out = hk.paged_decode_attn(g(batch["q"]), g(paged["K_pool"]), g(paged["V_pool"]), g(paged["act_pool"]),
                               g(paged["block_table"]), g(paged["seq_len"]), bt, lp, n_act_used=paged["n_act_used"],
                               absorbed=absorbed, **_prefix_sums(seq_len))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    # the oracle walks the same tables; on the big case only a sample of the requests
    sample = list(range(B)) if B <= 8 else ([0, 1, B // 2, B - 1] if d < 8192 else [0, B - 1])
    ref = pgo.paged_decode_attn(batch["q"][sample], paged["K_pool"], paged["V_pool"], paged["act_pool"],
                                paged["block_table"][sample], paged["seq_len"][sample], bt,
                                p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
    _check("out", out[sample], ref)
    for b in range(B):
        if seq_len[b] == 0:
            assert (out[b] == 0).all()


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [False, True], ids=["regenerating", "absorbed"])
def test_paged_decode_without_a_kv_pool(absorbed):
    """Every block a checkpoint block and no KV pool at all (P_kv == 0, NULL pools)."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("no_kv_pool", 512, 8, 4, 150, 0.5, 53)
    p, batch = _context(cfg, 6)
    seq_len = [150, 33, 64, 1]
    bt = 32
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, 1.0, seed=8)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    out = hk.paged_decode_attn(g(batch["q"]), None, None, g(paged["act_pool"]), g(paged["block_table"]), g(paged["seq_len"]), bt, lp,
                               n_act_used=paged["n_act_used"], absorbed=absorbed, **_prefix_sums(seq_len))
    torch.cuda.synchronize()
    ref = pgo.paged_decode_attn(batch["q"], paged["K_pool"], paged["V_pool"], paged["act_pool"], paged["block_table"],
                                paged["seq_len"], bt, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], cfg.n_heads)
    _check("out", out.cpu().numpy(), ref)


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [False, True], ids=["regenerating", "absorbed"])
def test_paged_decode_replayed_from_a_graph(absorbed):
    """The paged step captured in a HIP graph (tables, prefix sums and workspace on the device, nothing allocated
    inside): every replay, with eager work and synchronisations in between and the inputs changed before the
    last one, equals the eager result.  The entry point without regeneration sizes its launch on the host and
    reads the number of cached tokens from the device, inside the graph."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("paged_graph", 512, 4, 5, 180, 0.5, 54)
    p, batch = _context(cfg, 9)
    seq_len = [180, 7, 64, 0, 131]
    bt = 16
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, [0.5, 1.0, 0.0, 0.5, 0.3], seed=10)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    lp = lp + (hk.prepare_layer(*lp, cfg.n_heads),)
    q, Kp, Vp, Ap = g(batch["q"]), g(paged["K_pool"]), g(paged["V_pool"]), g(paged["act_pool"])
    tb, sl = g(paged["block_table"]), g(paged["seq_len"])
    cu = g(np.concatenate([[0], np.cumsum(seq_len)]).astype(np.int64))
    total = int(sum(seq_len))
    shape = hk.make_shape(cfg.d, cfg.n_heads)
    cache = hk.make_paged_cache(Kp, Vp, Ap, tb, sl, cu, total, bt, paged["n_act_used"])
    size_fn = hk.lib().hk_paged_absorbed_workspace_bytes if absorbed else hk.lib().hk_paged_workspace_bytes
    ws = hk.new_workspace(int(size_fn(ctypes.byref(shape), cfg.B, ctypes.byref(cache))))
    out = torch.empty(cfg.B, cfg.n_heads, cfg.head_dim, dtype=torch.float16, device="cuda")
    run = lambda stream: hk.paged_decode_attn(q, Kp, Vp, Ap, tb, sl, bt, lp, n_act_used=paged["n_act_used"], out=out,
                                              absorbed=absorbed, cu_tokens=cu, total_tokens=total, workspace=ws, stream=stream)
    run(None)                                                  # eager (also sets kernel attributes before the capture)
    torch.cuda.synchronize()
    eager = out.clone()
    ref = pgo.paged_decode_attn(batch["q"], paged["K_pool"], paged["V_pool"], paged["act_pool"], paged["block_table"],
                                paged["seq_len"], bt, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], cfg.n_heads)
    _check("eager", eager.cpu().numpy(), ref)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(torch.cuda.current_stream())
    for i in range(3):
        out.fill_(7.0)
        ws.view(torch.uint8).fill_(0xff)                       # stale scratch must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from the eager result" % i
        (q.float().sum() + Kp.float().sum()).item()            # eager work between the replays
    q.mul_(0.5)                                                # new inputs, same addresses
    run(None)
    torch.cuda.synchronize()
    eager2 = out.clone()
    out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager2)
    assert not torch.equal(eager2, eager)


def test_qkv_current_paged_rejects_bad_arguments():
    """Every check of hk_qkv_current_paged runs on the host before a launch: no GPU is touched here."""
    FAKE = 0x10000
    ok = hk.make_shape(768, 12)
    lp = hk.hk_layer_params(FAKE, FAKE, FAKE, FAKE, None)

    def cache(**kw):
        f = dict(K_pool=FAKE, V_pool=FAKE, act_pool=FAKE, block_table=FAKE, seq_len=FAKE, cu_tokens=None,
                 total_tokens=0, P_kv=8, P_act=8, n_act_used=0, block_tokens=16, max_blocks=8)
        f.update(kw)
        return hk.hk_paged_cache(**f)

    def call(shape=ok, x=FAKE, B=4, c=None, lp=lp, Wq=FAKE, bq=FAKE, q=FAKE, ws=FAKE, n=1 << 40, null_cache=False, mask=None):
        c = c or cache()
        return hk.lib().hk_qkv_current_paged(ctypes.byref(shape), x, B, ctypes.byref(lp), Wq, bq, q,
                                             None if null_cache else ctypes.byref(c), mask, ws, n, None)

    assert call(null_cache=True) == hk.HK_ERR_NULL
    assert call(c=cache(block_tokens=24)) == hk.HK_ERR_SHAPE and call(c=cache(block_tokens=8)) == hk.HK_ERR_SHAPE
    assert call(c=cache(max_blocks=0)) == hk.HK_ERR_SHAPE and call(c=cache(P_kv=-1)) == hk.HK_ERR_SHAPE
    assert call(shape=hk.make_shape(768, 11)) == hk.HK_ERR_SHAPE
    assert call(c=cache(block_table=None)) == hk.HK_ERR_NULL and call(c=cache(seq_len=None)) == hk.HK_ERR_NULL
    assert call(c=cache(K_pool=None)) == hk.HK_ERR_NULL and call(c=cache(act_pool=None)) == hk.HK_ERR_NULL
    assert call(c=cache(P_kv=0, K_pool=None, V_pool=None), x=None) == hk.HK_ERR_NULL     # no KV pool is fine, no input is not
    assert call(x=None) == hk.HK_ERR_NULL and call(q=None) == hk.HK_ERR_NULL and call(Wq=None) == hk.HK_ERR_NULL
    assert call(c=cache(seq_len=FAKE + 2)) == hk.HK_ERR_ALIGN and call(c=cache(K_pool=FAKE + 8)) == hk.HK_ERR_ALIGN
    assert call(n=hk.hk_qkv_workspace_bytes(ok, 4) - 1) == hk.HK_ERR_WORKSPACE
    assert call(B=0, x=None) == hk.HK_OK
    assert call(mask=FAKE + 2) == hk.HK_ERR_ALIGN and call(mask=FAKE, x=None) == hk.HK_ERR_NULL
    bf = hk.make_shape(768, 12, dtype=hk.HK_DTYPE_BF16)
    assert call(shape=bf, c=cache(block_tokens=24)) == hk.HK_ERR_SHAPE and call(shape=bf, x=None) == hk.HK_ERR_NULL


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("case", [("mixed", 768, 12, 7, 16, True), ("rows130", 512, 8, 130, 32, True),
                                  ("no_kv_pool", 512, 4, 5, 16, False)], ids=lambda c: c[0])
def test_qkv_current_paged_writes_the_row_its_table_names(case, dtype):
    """hk_qkv_current_paged: q for every request; the token's K/V rows land in the row of the KV block its table
    entry names, or its layer input in the row of the ACT block; nothing else in the pools changes; a request
    without tokens and entries outside the pools are not written; the same q as hk_qkv_current."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    name, d, H, B, bt, with_kv = case
    print("case", case, dtype, flush=True)
    dh = d // H
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float16
    cfg = synth.LayerConfig(name, d, H, B, 8, 0.5, 57)
    p, c = synth.make_params(cfg), synth.make_current_token(cfg)
    g, h = {}, {}
    for k, v in {**p, **c}.items():
        t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(tdt)
        g[k], h[k] = t.cuda(), t.float().numpy().astype(np.float64)
    rng = np.random.default_rng(58)
    max_blocks = 6
    P_kv, P_act = (B + 3, B + 2) if with_kv else (0, B + 2)
    seq_len = rng.integers(1, max_blocks * bt + 1, B).astype(np.int32)
    seq_len[0] = max_blocks * bt                           # the last row of the last block
    if B > 2:
        seq_len[1] = 0                                     # no token: nothing is written for it
        seq_len[2] = bt + 1                                # the first row of a fresh block
    table = np.full((B, max_blocks), 0x7fffffff, dtype=np.int32)
    kv_ids, act_ids = rng.permutation(max(P_kv, 1)), rng.permutation(P_act)
    kinds = []
    for b in range(B):
        t = int(seq_len[b]) - 1
        is_act = (not with_kv) or bool(rng.random() < 0.5)
        kinds.append(is_act)
        if t >= 0:
            table[b, t // bt] = ~int(act_ids[b % P_act]) if is_act else int(kv_ids[b % P_kv])
    if B > 4 and with_kv:
        table[4, (int(seq_len[4]) - 1) // bt] = P_kv + 5   # a KV entry outside the pool: not written
    Kp = torch.full((max(P_kv, 1), H, bt, dh), 7.0, dtype=tdt, device="cuda")
    Vp = torch.full((max(P_kv, 1), H, bt, dh), -7.0, dtype=tdt, device="cuda")
    Ap = torch.full((P_act, bt, d), 3.0, dtype=tdt, device="cuda")
    q = hk.qkv_current_paged(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H,
                             Kp if with_kv else None, Vp if with_kv else None, Ap,
                             torch.from_numpy(table).cuda(), torch.from_numpy(seq_len).cuda(), bt)
    torch.cuda.synchronize()
    rq, rk, rv = ho.qkv_current(h["x_cur"], h["ln_w"], h["ln_b"], h["Wq"], h["bq"], h["Wkv"], h["bkv"], H)
    tol_abs = (lambda ref: 2.0 ** -7 * np.abs(ref).max()) if dtype == "bf16" else (lambda ref: MAX_ABS)

    def check(name_, got, ref):
        got = got.float().cpu().numpy().astype(np.float64)
        err, rel = np.abs(got - ref).max(), np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
        print("%s: max_abs=%.3e rel_l2=%.3e" % (name_, err, rel), flush=True)
        assert err <= tol_abs(ref) and rel <= REL_L2, (name_, err, rel)

    check("q", q, rq)
    Kexp = torch.full_like(Kp, 7.0); Vexp = torch.full_like(Vp, -7.0); Aexp = torch.full_like(Ap, 3.0)
    written_k, written_a = [], []
    for b in range(B):
        t = int(seq_len[b]) - 1
        if t < 0:
            continue
        e, r = int(table[b, t // bt]), t % bt
        if e >= 0 and with_kv and e < P_kv:
            written_k.append((b, e, r))
        elif e < 0 and ~e < P_act:
            written_a.append((b, ~e, r))
    for b, e, r in written_k:
        check("k[%d]" % b, Kp[e, :, r], rk[b]); check("v[%d]" % b, Vp[e, :, r], rv[b])
        Kexp[e, :, r] = Kp[e, :, r]; Vexp[e, :, r] = Vp[e, :, r]
    for b, e, r in written_a:
        assert torch.equal(Ap[e, r], g["x_cur"][b])        # the checkpoint is the layer input, bit for bit
        Aexp[e, r] = Ap[e, r]
    assert torch.equal(Kp, Kexp) and torch.equal(Vp, Vexp) and torch.equal(Ap, Aexp)   # nothing else was touched
    assert len(written_a) > 0 and (len(written_k) > 0 or not with_kv)
    q2 = hk.qkv_current(g["x_cur"], g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"], g["Wq"], g["bq"], H)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [False, True], ids=["regenerating", "absorbed"])
def test_paged_decode_step_with_current_token(absorbed):
    """The whole paged decode step of a layer from this library: QKV generation of the input tokens with the
    write-back into the blocks their tables name (hk_qkv_current_paged), then the attention of the generated
    queries over the paged context including those tokens; against the oracle given the finished pools."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("paged_step", 768, 12, 6, 120, 0.5, 59)
    H, d, bt = cfg.n_heads, cfg.d, 16
    p, batch = _context(cfg, 15)
    cur = synth.make_current_token(cfg)
    seq_len = [120, 1, 17, 64, 0, 99]
    oq, ok_, ov = ho.qkv_current(cur["x_cur"], p["ln_w"], p["ln_b"], cur["Wq"], cur["bq"], p["Wkv"], p["bkv"], H)
    for b, n in enumerate(seq_len):                        # the input token is the last token of its request
        if n > 0:
            batch["act_full"][b, n - 1] = cur["x_cur"][b]
            batch["K_full"][b, :, n - 1] = ok_[b].astype(np.float16)
            batch["V_full"][b, :, n - 1] = ov[b].astype(np.float16)
    batch["q"] = oq.astype(np.float16)
    paged = synth.scatter_into_blocks(cfg, batch, seq_len, bt, [0.5, 0.0, 1.0, 0.5, 0.5, 0.4], seed=16)
    ref = pgo.paged_decode_attn(batch["q"], paged["K_pool"], paged["V_pool"], paged["act_pool"], paged["block_table"],
                                paged["seq_len"], bt, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    Kp, Vp, Ap = g(paged["K_pool"]), g(paged["V_pool"]), g(paged["act_pool"])
    for b, n in enumerate(seq_len):                        # the pools before the step: the input token's row is not there yet
        if n > 0:
            e, r = int(paged["block_table"][b, (n - 1) // bt]), (n - 1) % bt
            if e >= 0:
                Kp[e, :, r] = 99.0; Vp[e, :, r] = -99.0
            else:
                Ap[~e, r] = 99.0
    tb, sl = g(paged["block_table"]), g(paged["seq_len"])
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    q = hk.qkv_current_paged(g(cur["x_cur"]), *lp, g(cur["Wq"]), g(cur["bq"]), H, Kp, Vp, Ap, tb, sl, bt)
    out = hk.paged_decode_attn(q, Kp, Vp, Ap, tb, sl, bt, lp, n_act_used=paged["n_act_used"], absorbed=absorbed,
                               **_prefix_sums(seq_len))
    torch.cuda.synchronize()
    _check("q", q.cpu().numpy(), oq)
    _check("out", out.cpu().numpy(), ref)
    assert (out[4] == 0).all()                             # the request without tokens


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [True, False], ids=["absorbed", "regenerating"])
def test_paged_decode_loop_replayed_from_one_graph(absorbed):
    """A device-resident decode loop: the block bookkeeping of the step (hk_paged_append: lengths, prefix sums, new
    blocks by the ratio rule), QKV generation with the paged write-back and the attention (with and without
    regeneration), captured ONCE in a HIP graph with total_tokens and n_act_used given as upper bounds, then
    replayed for successive decode steps; the host only writes the new input rows in between.  Every step is
    checked against the oracles: tables, lengths and counters bit for bit, q and the output within tolerance on
    the pools as they then are."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("paged_loop", 512, 8, 4, 64, 0.5, 60)
    H, d, B, bt, max_blocks, steps = cfg.n_heads, cfg.d, cfg.B, 16, 6, 4
    p, batch = _context(cfg, 17)
    cur = synth.make_current_token(cfg)
    lens0 = [30, 16, 0, 47]                                # the second request starts a new block at once, the third is empty
    paged = synth.scatter_into_blocks(cfg, batch, lens0, bt, 0.5, seed=18)
    n_kv0, n_act0 = paged["K_pool"].shape[0], paged["act_pool"].shape[0]
    # room for the blocks the loop will open; they are handed out on the device by hk_paged_append (host ratio 1:1),
    # after the blocks the initial context occupies (its KV blocks are scattered over the whole initial pool)
    extra = B * 2
    Kp = np.concatenate([paged["K_pool"], np.zeros((extra,) + paged["K_pool"].shape[1:], np.float16)])
    Vp = np.concatenate([paged["V_pool"], np.zeros((extra,) + paged["V_pool"].shape[1:], np.float16)])
    Ap = np.concatenate([paged["act_pool"], np.zeros((extra,) + paged["act_pool"].shape[1:], np.float16)])
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    table[:, :paged["block_table"].shape[1]] = paged["block_table"]
    counters = np.asarray([n_kv0, paged["n_act_used"], 0, 0], np.int32)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    Kg, Vg, Ag, tb = g(Kp), g(Vp), g(Ap), g(table)
    sl, cn = g(np.asarray(lens0, np.int32)), g(counters)
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    lp = lp + (hk.prepare_layer(*lp, H),)
    Wq, bq = g(cur["Wq"]), g(cur["bq"])
    x = torch.zeros(B, d, dtype=torch.float16, device="cuda")
    q = torch.empty(B, H, d // H, dtype=torch.float16, device="cuda")
    out = torch.empty_like(q)
    bound = B * max_blocks * bt                            # more tokens than the loop will ever hold
    cu_dev = torch.zeros(B + 1, dtype=torch.int64, device="cuda")     # kept up to date on the device (the form without
    shape = hk.make_shape(d, H)                                        # regeneration does not even read it)
    cache = hk.make_paged_cache(Kg, Vg, Ag, tb, sl, cu_dev, bound, bt, Ag.shape[0])
    ws_q = hk.new_workspace(hk.hk_qkv_workspace_bytes(shape, B))
    size_fn = hk.lib().hk_paged_absorbed_workspace_bytes if absorbed else hk.lib().hk_paged_workspace_bytes
    ws_a = hk.new_workspace(int(size_fn(ctypes.byref(shape), B, ctypes.byref(cache))))

    grew = torch.full((B,), -1, dtype=torch.int32, device="cuda")

    def step(stream):
        hk.paged_append(tb, sl, cu_dev, cn, Kg.shape[0], Ag.shape[0], bt, 1, 1, stream=stream, grew=grew)
        hk.qkv_current_paged(x, *lp[:4], Wq, bq, H, Kg, Vg, Ag, tb, sl, bt, q_out=q, workspace=ws_q, stream=stream,
                             store_mask=grew)
        hk.paged_decode_attn(q, Kg, Vg, Ag, tb, sl, bt, lp, n_act_used=Ag.shape[0], out=out, absorbed=absorbed,
                             cu_tokens=cu_dev, total_tokens=bound, workspace=ws_a, stream=stream)

    rng = np.random.default_rng(19)
    graph = None
    for s in range(steps):
        x_np = rng.standard_normal((B, d)).astype(np.float16)
        x.copy_(g(x_np))                                   # the only thing the host does between the steps
        torch.cuda.synchronize()
        ref_table, ref_lens, ref_cu, ref_cnt = pgo.paged_append(tb.cpu().numpy(), sl.cpu().numpy(), cn.cpu().numpy(), None, bt,
                                                                Kg.shape[0], Ag.shape[0], 1, 1)
        if graph is None:
            saved = [t.clone() for t in (Kg, Vg, Ag, tb, sl, cn, cu_dev)]
            step(None)                                     # eager once (kernel attributes), then undone
            torch.cuda.synchronize()
            for t, c in zip((Kg, Vg, Ag, tb, sl, cn, cu_dev), saved):
                t.copy_(c)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step(torch.cuda.current_stream())
        out.fill_(5.0)
        graph.replay()
        torch.cuda.synchronize()
        lens, table = sl.cpu().numpy(), tb.cpu().numpy()
        assert np.array_equal(table, ref_table) and np.array_equal(lens, ref_lens) and np.array_equal(cn.cpu().numpy(), ref_cnt)
        assert np.array_equal(cu_dev.cpu().numpy(), ref_cu) and (grew == 1).all()
        oq, _, _ = ho.qkv_current(x_np, p["ln_w"], p["ln_b"], cur["Wq"], cur["bq"], p["Wkv"], p["bkv"], H)
        ref = pgo.paged_decode_attn(q.cpu().numpy(), Kg.cpu().numpy(), Vg.cpu().numpy(), Ag.cpu().numpy(), table, lens, bt,
                                    p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
        _check("q step %d" % s, q.cpu().numpy(), oq)
        _check("out step %d" % s, out.cpu().numpy(), ref)
        for b in range(B):                                 # the token is where the table says, bit for bit when a checkpoint
            e, r = int(table[b, (lens[b] - 1) // bt]), (lens[b] - 1) % bt
            if e < 0:
                assert torch.equal(Ag[~e, r], x[b])


# ------------------------------------------------------------------ the bookkeeping of a decode step (Eq. 11)
def test_paged_append_oracle_pins():
    """The append oracle against what the paper and arithmetic fix: the worked example of Sec. 4.3 (host ratio 3:1,
    a request with five checkpoint and two KV blocks opens a checkpoint block); over a long run every request's
    checkpoint share stays within one block of the host share; blocks are handed out once each, in order, inside
    their pools; lengths grow by one; a full table row and an exhausted pool stop a request and are counted."""
    bt = 16
    table = np.full((1, 16), 0x7fffffff, np.int32)
    table[0, :7] = [~0, ~1, 0, ~2, ~3, 1, ~4]              # five checkpoint blocks, two KV blocks, all full
    t, l, cu, c = pgo.paged_append(table, [7 * bt], [2, 5, 0, 0], None, bt, 100, 100, 3, 1)
    assert t[0, 7] == ~5 and l[0] == 7 * bt + 1 and list(c) == [2, 6, 0, 0] and list(cu) == [0, 7 * bt + 1]
    # a long run from empty: ratios, uniqueness, bounds, lengths
    B, max_blocks, act_host, kv_host = 5, 40, 3, 2
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    lens, cnt = np.zeros(B, np.int32), np.zeros(4, np.int32)
    rng = np.random.default_rng(3)
    for step in range(30 * bt):
        active = (rng.random(B) < 0.8).astype(np.int32)
        table2, lens2, cu, cnt = pgo.paged_append(table, lens, cnt, active, bt, 1000, 1000, act_host, kv_host)
        assert np.array_equal(lens2, lens + active) and np.array_equal(cu[1:], np.cumsum(lens2)) and cu[0] == 0
        table, lens = table2, lens2
        for b in range(B):
            n = (int(lens[b]) + bt - 1) // bt
            n_act = int((table[b, :n] < 0).sum())
            assert abs(n_act * (act_host + kv_host) - act_host * n) <= act_host + kv_host     # within one block of the share
            assert (table[b, n:] == 0x7fffffff).all()
    kv = sorted(int(e) for e in table.ravel() if 0 <= e < 0x7fffffff)
    act = sorted(int(~e) for e in table.ravel() if e < 0)
    assert kv == list(range(cnt[0])) and act == list(range(cnt[1])) and cnt[2] == 0
    # a full row, and an exhausted pool
    t, l, _, c, gr = pgo.paged_append(np.zeros((1, 2), np.int32), [2 * bt], [2, 0, 0, 0], None, bt, 10, 10, 1, 1, with_grew=True)
    assert l[0] == 2 * bt and c[2] == 1 and list(gr) == [0]
    # which requests took their token: the active ones that were not stopped
    _, l, _, _, gr = pgo.paged_append(np.zeros((3, 2), np.int32), [2 * bt, 5, 7], [3, 0, 0, 0], [1, 0, 1], bt, 10, 10, 1, 1,
                                      with_grew=True)
    assert list(gr) == [0, 0, 1] and list(l) == [2 * bt, 5, 8]
    t, l, _, c = pgo.paged_append(np.full((2, 4), 0x7fffffff, np.int32), [0, 0], [0, 1, 0, 0], None, bt, 10, 1, 1, 0)
    assert list(l) == [0, 0] and c[2] == 2 and c[1] == 1   # only checkpoint blocks are due and their pool is full


def test_paged_append_rejects_bad_arguments():
    FAKE = 0x10000
    def call(table=FAKE, sl=FAKE, cu=FAKE, cnt=FAKE, active=None, B=4, max_blocks=8, bt=16, P_kv=8, P_act=8, a=3, k=1, grew=None):
        return hk.lib().hk_paged_append(table, sl, cu, cnt, active, grew, B, max_blocks, bt, P_kv, P_act, a, k, None)
    assert call(bt=24) == hk.HK_ERR_SHAPE and call(bt=8) == hk.HK_ERR_SHAPE and call(max_blocks=0) == hk.HK_ERR_SHAPE
    assert call(a=0, k=0) == hk.HK_ERR_SHAPE and call(a=-1) == hk.HK_ERR_SHAPE and call(B=65536) == hk.HK_ERR_SHAPE
    assert call(P_kv=-1) == hk.HK_ERR_SHAPE
    assert call(table=None) == hk.HK_ERR_NULL and call(sl=None) == hk.HK_ERR_NULL and call(cu=None) == hk.HK_ERR_NULL
    assert call(cnt=None) == hk.HK_ERR_NULL
    assert call(cu=FAKE + 4) == hk.HK_ERR_ALIGN and call(active=FAKE + 2) == hk.HK_ERR_ALIGN and call(grew=FAKE + 2) == hk.HK_ERR_ALIGN
    assert call(B=0, table=None) == hk.HK_OK


@pytest.mark.gpu
@pytest.mark.parametrize("case", [("small", 5, 12, 16, 40, 40, 3, 1, 60), ("many_requests", 700, 6, 16, 900, 2000, 2, 3, 40),
                                  ("tight_pools", 9, 10, 32, 7, 11, 1, 1, 200), ("only_act", 4, 8, 16, 0, 30, 1, 0, 50)],
                         ids=lambda c: c[0])
def test_paged_append_matches_oracle(case):
    """hk_paged_append step by step against the oracle: tables, lengths, prefix sums and counters, bit for bit
    (integer work), with random active masks, from empty requests, through full table rows and exhausted pools."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    name, B, max_blocks, bt, P_kv, P_act, act_host, kv_host, steps = case
    print("case", case, flush=True)
    rng = np.random.default_rng(7)
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    lens = np.zeros(B, np.int32)
    cnt = np.zeros(4, np.int32)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    tb, sl, cn = g(table), g(lens), g(cnt)
    cu = torch.full((B + 1,), -1, dtype=torch.int64, device="cuda")
    for s in range(steps):
        active = None if s % 5 == 0 else (rng.random(B) < 0.7).astype(np.int32)
        # a few big strides so that rows fill up and pools run dry within the test
        if s == 3:
            bump = (rng.integers(0, max_blocks, B) * bt).astype(np.int32)
            lens_np = sl.cpu().numpy()
            # only lengths at a block boundary may jump (their tables stay consistent: whole blocks are laid out by hand)
            table_np, cnt_np = tb.cpu().numpy(), cn.cpu().numpy()
            for b in range(B):
                if lens_np[b] % bt == 0 and bump[b] > 0 and lens_np[b] + bump[b] <= max_blocks * bt:
                    i0 = lens_np[b] // bt
                    for i in range(i0, i0 + bump[b] // bt):
                        if cnt_np[1] < P_act:
                            table_np[b, i] = ~int(cnt_np[1]); cnt_np[1] += 1
                        elif cnt_np[0] < P_kv:
                            table_np[b, i] = int(cnt_np[0]); cnt_np[0] += 1
                        else:
                            break
                    else:
                        lens_np[b] += bump[b]
            tb.copy_(g(table_np)); sl.copy_(g(lens_np)); cn.copy_(g(cnt_np))
        ref_t, ref_l, ref_cu, ref_c, ref_g = pgo.paged_append(tb.cpu().numpy(), sl.cpu().numpy(), cn.cpu().numpy(), active, bt,
                                                              P_kv, P_act, act_host, kv_host, with_grew=True)
        grew = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        hk.paged_append(tb, sl, cu, cn, P_kv, P_act, bt, act_host, kv_host, active=None if active is None else g(active),
                        grew=grew)
        torch.cuda.synchronize()
        assert np.array_equal(grew.cpu().numpy(), ref_g), "grew, step %d" % s
        assert np.array_equal(tb.cpu().numpy(), ref_t), "table, step %d" % s
        assert np.array_equal(sl.cpu().numpy(), ref_l), "lengths, step %d" % s
        assert np.array_equal(cu.cpu().numpy(), ref_cu), "prefix sums, step %d" % s
        assert np.array_equal(cn.cpu().numpy(), ref_c), "counters, step %d" % s
    assert name != "tight_pools" or int(cn[2]) > 0          # the case did run into its limits


@pytest.mark.gpu
@pytest.mark.parametrize("absorbed", [False, True], ids=["regenerating", "absorbed"])
@pytest.mark.parametrize("lens", [[2], [40], [1, 0, 33]], ids=["len2", "len40", "three"])
def test_paged_decode_with_a_loose_token_bound(lens, absorbed):
    """total_tokens may be any upper bound of the tokens the device finds (a graph captured for a long context
    serves a short one): with H * tokens far below the wavefronts the bound launches, the wavefronts past the
    device's total must drop out and the merge must read written partials only.  Bound = 4096 tokens against
    2 .. 40 real ones, 72 heads, workspace filled with NaN patterns beforehand."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    H, dh, bt, max_blocks = 72, 128, 16, 256
    B = len(lens)
    cfg = synth.LayerConfig("loose_bound", H * dh, H, B, max(lens), 0.5, 61)
    p, batch = _context(cfg, 21)
    paged = synth.scatter_into_blocks(cfg, batch, lens, bt, 0.5, seed=22)
    g = lambda x: None if x is None or x.shape[0] == 0 else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    table[:, :paged["block_table"].shape[1]] = paged["block_table"]
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    q, Kp, Vp, Ap = g(batch["q"]), g(paged["K_pool"]), g(paged["V_pool"]), g(paged["act_pool"])
    tb, sl = g(table), g(paged["seq_len"])
    cu = g(np.concatenate([[0], np.cumsum(lens)]).astype(np.int64))
    bound = 4096
    shape = hk.make_shape(cfg.d, H)
    cache = hk.make_paged_cache(Kp, Vp, Ap, tb, sl, cu, bound, bt, paged["n_act_used"])
    size_fn = hk.lib().hk_paged_absorbed_workspace_bytes if absorbed else hk.lib().hk_paged_workspace_bytes
    ws = hk.new_workspace(int(size_fn(ctypes.byref(shape), B, ctypes.byref(cache))))
    ws.fill_(0xff)                                             # fp32 NaN in every partial slot
    out = hk.paged_decode_attn(q, Kp, Vp, Ap, tb, sl, bt, lp, n_act_used=paged["n_act_used"], absorbed=absorbed,
                               cu_tokens=cu, total_tokens=bound, workspace=ws)
    torch.cuda.synchronize()
    ref = pgo.paged_decode_attn(batch["q"], paged["K_pool"], paged["V_pool"], paged["act_pool"], paged["block_table"],
                                paged["seq_len"], bt, p["ln_w"], p["ln_b"], p["Wkv"], p["bkv"], H)
    _check("out", out.cpu().numpy(), ref)


@pytest.mark.gpu
def test_paged_decode_loop_leaves_requests_that_did_not_grow_alone():
    """A decode loop in which one request is inactive and another cannot grow (its table row is full): the
    `grew` array of hk_paged_append masks the write-back of hk_qkv_current_paged, so the last cached token of
    those requests, a KV row or a checkpoint, stays as it was; the requests that grew get their rows."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU path")
    cfg = synth.LayerConfig("paged_mask", 512, 8, 5, 48, 0.5, 62)
    H, d, B, bt, max_blocks = cfg.n_heads, cfg.d, cfg.B, 16, 3
    p, batch = _context(cfg, 23)
    cur = synth.make_current_token(cfg)
    lens0 = [48, 20, 33, 48, 7]                            # requests 0 and 3 fill their table rows (3 blocks of 16)
    paged = synth.scatter_into_blocks(cfg, batch, lens0, bt, [0.0, 0.5, 0.5, 1.0, 0.5], seed=24)
    g = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    extra = 4
    Kg = g(np.concatenate([paged["K_pool"], np.zeros((extra,) + paged["K_pool"].shape[1:], np.float16)]))
    Vg = g(np.concatenate([paged["V_pool"], np.zeros((extra,) + paged["V_pool"].shape[1:], np.float16)]))
    Ag = g(np.concatenate([paged["act_pool"], np.zeros((extra,) + paged["act_pool"].shape[1:], np.float16)]))
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    table[:, :paged["block_table"].shape[1]] = paged["block_table"]
    tb, sl = g(table), g(np.asarray(lens0, np.int32))
    cn = g(np.asarray([paged["K_pool"].shape[0], paged["n_act_used"], 0, 0], np.int32))
    cu = torch.zeros(B + 1, dtype=torch.int64, device="cuda")
    active = g(np.asarray([1, 0, 1, 1, 1], np.int32))      # request 1 sits this step out
    grew = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    lp = tuple(g(p[k]) for k in ("ln_w", "ln_b", "Wkv", "bkv"))
    K0, V0, A0 = Kg.clone(), Vg.clone(), Ag.clone()
    hk.paged_append(tb, sl, cu, cn, Kg.shape[0], Ag.shape[0], bt, 1, 1, active=active, grew=grew)
    q = hk.qkv_current_paged(g(cur["x_cur"]), *lp, g(cur["Wq"]), g(cur["bq"]), H, Kg, Vg, Ag, tb, sl, bt, store_mask=grew)
    torch.cuda.synchronize()
    assert grew.cpu().tolist() == [0, 0, 1, 0, 1] and int(cn[2]) == 2
    lens, table = sl.cpu().numpy(), tb.cpu().numpy()
    assert lens.tolist() == [48, 20, 34, 48, 8]
    oq, ok_, ov = ho.qkv_current(cur["x_cur"], p["ln_w"], p["ln_b"], cur["Wq"], cur["bq"], p["Wkv"], p["bkv"], H)
    _check("q", q.cpu().numpy(), oq)                       # every request gets its query
    Kexp, Vexp, Aexp = K0.clone(), V0.clone(), A0.clone()
    for b in (2, 4):                                       # only the rows of the requests that grew may differ
        e, r = int(table[b, (lens[b] - 1) // bt]), (lens[b] - 1) % bt
        if e >= 0:
            _check("k[%d]" % b, Kg[e, :, r].cpu().numpy(), ok_[b]); _check("v[%d]" % b, Vg[e, :, r].cpu().numpy(), ov[b])
            Kexp[e, :, r] = Kg[e, :, r]; Vexp[e, :, r] = Vg[e, :, r]
        else:
            assert torch.equal(Ag[~e, r], g(cur["x_cur"])[b])
            Aexp[~e, r] = Ag[~e, r]
    assert torch.equal(Kg, Kexp) and torch.equal(Vg, Vexp) and torch.equal(Ag, Aexp)
    # without the mask the same call does overwrite the last cached token of the three others: the hazard is real
    hk.qkv_current_paged(g(cur["x_cur"]), *lp, g(cur["Wq"]), g(cur["bq"]), H, Kg, Vg, Ag, tb, sl, bt)
    torch.cuda.synchronize()
    assert not (torch.equal(Kg, Kexp) and torch.equal(Ag, Aexp))
