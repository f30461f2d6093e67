"""Timing of the entry points beside the benchmark's path (bench.py times the hybrid step itself):

    python -m paper_2501_01792_amd.measure qkv   [--config opt6.7b] [--iters 20]
    python -m paper_2501_01792_amd.measure paged [--config opt66b] [--block-tokens 16] [--act-fraction 0.0] [--ragged] [--absorbed] [--graph]

    python -m paper_2501_01792_amd.measure loop  [--config opt6.7b] [--block-tokens 16] [--act-fraction 0.5] [--ragged] [--iters 20]
    python -m paper_2501_01792_amd.measure overlap [--config opt6.7b] [--iters 20]
    python -m paper_2501_01792_amd.measure gemm    [--config opt66b] [--iters 6]
    python -m paper_2501_01792_amd.measure read    [--config opt66b] [--iters 5]

Each prints one JSON line.  Inputs are drawn on the GPU with the scales of the benchmark recipe (timing only;
parity is the tests' business).  ``qkv`` measures hk_qkv_current (Sec. 4.2.2, QKV generation of the current
token) COLD: the weights of one layer fit in the 256 MB last-level cache, which a real decoder of dozens of
layers would have evicted by the time a layer comes round again, so a 512 MiB buffer is read between calls.
``paged`` measures hk_paged_decode_attn (Sec. 4.1, 5.1: block table, ragged requests) on the workload's
B, H, L with blocks of ``--block-tokens`` tokens scattered over the pools in random order.  ``loop`` measures one
decode step of a layer on that paged cache as a serving loop would run it: hk_paged_append, hk_qkv_current_paged and
hk_paged_decode_attn_absorbed captured once in a HIP graph and replayed, the context growing by a token per replay.
``overlap`` measures hk_hybrid_decode_attn_two_stream (the attention over the cached segment on a side stream beside the
regeneration) against the single-stream step, with the projection kernel on all compute units and on all but 8, 16, 32.
``gemm`` measures hk_regen_kv (LayerNorm statistics + projection with bias and head-split stores) on the workload's
regeneration GEMM (all of its tokens as checkpoints) alternately with a plain library GEMM on the same operands
(torch.addmm, i.e. hipBLASLt: no LayerNorm, row-major output), as a comparator for what this GPU sustains on the shape.
``read`` measures how fast the workload's checkpoint rows stream from HBM with the load structure of the streaming
kernels (32 rows per wavefront, 20 KiB in flight each) for four shapes of one load instruction, plain and non-temporal.
"""
import argparse
import json
import sys

import numpy as np


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def measure_qkv(args):
    import torch
    from . import binding as hk, synth
    cfg = synth.CONFIGS[args.config]
    B, d, H, dh = cfg.B, cfg.d, cfg.n_heads, cfg.head_dim
    f16 = torch.float16
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen, device="cuda") * std + mean).to(f16)
    x = rn(B, d)
    Wq, bq, Wkv, bkv = rn(d, d, std=0.02), rn(d, std=0.01), rn(2 * d, d, std=0.02), rn(2 * d, std=0.01)
    ln_w, ln_b = rn(d, std=0.02, mean=1.0), rn(d, std=0.02)
    K = torch.empty(B, H, 4, dh, device="cuda", dtype=f16)
    V = torch.empty_like(K)
    q = torch.empty(B, H, dh, device="cuda", dtype=f16)
    ws = hk.new_workspace(hk.hk_qkv_workspace_bytes(hk.make_shape(d, H), B))
    flush = torch.empty(1 << 29, dtype=torch.uint8, device="cuda").fill_(1)
    out = {}
    for name, with_kv in (("q_k_v", True), ("q_only", False)):
        call = lambda: hk.qkv_current(x, ln_w, ln_b, Wkv, bkv, Wq, bq, H, q_out=q, K_dst=K if with_kv else None,
                                      V_dst=V if with_kv else None, tok_pos=1, workspace=ws)
        for _ in range(3):
            call()
        ts = []
        for _ in range(args.iters):
            flush.view(torch.int32).max()                      # evicts the weights from the last-level cache
            e0, e1 = _events(torch)
            e0.record(); call(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ms = float(np.mean(ts))
        nbytes = (6 if with_kv else 2) * d * d                 # one pass over the fp16 weights
        out[name] = {"ms": ms, "min_ms": float(np.min(ts)), "weight_bytes": nbytes, "GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / 8000.0}
    print(json.dumps({"entry": "hk_qkv_current", "workload": "%s: B=%d d=%d H=%d, cold" % (cfg.name, B, d, H),
                      "iters": args.iters, "result": out}))
    return 0


def measure_paged(args):
    import torch
    from . import binding as hk, synth
    cfg = synth.CONFIGS[args.config]
    B, d, H, dh, L, bt = cfg.B, cfg.d, cfg.n_heads, cfg.head_dim, cfg.L, args.block_tokens
    f16 = torch.float16
    rng = np.random.default_rng(cfg.seed)
    lens = rng.integers(L // 2, L + 1, B) if args.ragged else np.full(B, L)
    nb = (lens + bt - 1) // bt
    total_blocks, max_blocks = int(nb.sum()), int(nb.max())
    kinds = rng.random(total_blocks) < args.act_fraction
    n_act = int(kinds.sum())
    n_kv = total_blocks - n_act
    table = np.zeros((B, max_blocks), np.int32)
    pa, pk = rng.permutation(max(n_act, 1)), rng.permutation(max(n_kv, 1))
    ia = ik = k = 0
    for b in range(B):
        for i in range(nb[b]):
            if kinds[k]:
                table[b, i] = ~int(pa[ia]); ia += 1
            else:
                table[b, i] = int(pk[ik]); ik += 1
            k += 1
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen, device="cuda") * std + mean).to(f16)
    kv_std = 0.02 * d ** 0.5
    Kp = torch.empty(max(n_kv, 1), H, bt, dh, device="cuda", dtype=f16)
    Vp = torch.empty_like(Kp)
    step = max(1, (1 << 28) // (H * bt * dh))
    for i in range(0, Kp.shape[0], step):                      # drawn in pieces: the fp32 temporaries stay small
        Kp[i:i + step] = rn(*Kp[i:i + step].shape, std=kv_std)
        Vp[i:i + step] = rn(*Vp[i:i + step].shape, std=kv_std)
    Ap = rn(max(n_act, 1), bt, d)
    q = rn(B, H, dh, std=kv_std)
    Wkv, bkv = rn(2 * d, d, std=0.02), rn(2 * d, std=0.01)
    ln_w, ln_b = rn(d, std=0.02, mean=1.0), rn(d, std=0.02)
    lp = (ln_w, ln_b, Wkv, bkv)
    lp = lp + (hk.prepare_layer(*lp, H),)
    tb, sl = torch.from_numpy(table).cuda(), torch.from_numpy(lens.astype(np.int32)).cuda()
    out = torch.empty(B, H, dh, device="cuda", dtype=f16)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)).cuda()   # the tables live on the device
    total = int(lens.sum())
    shape = hk.make_shape(d, H)
    cache = hk.make_paged_cache(Kp if n_kv else None, Vp if n_kv else None, Ap if n_act else None, tb, sl, cu, total, bt, n_act)
    size_fn = hk.lib().hk_paged_absorbed_workspace_bytes if args.absorbed else hk.lib().hk_paged_workspace_bytes
    import ctypes
    ws = hk.new_workspace(int(size_fn(ctypes.byref(shape), B, ctypes.byref(cache))))
    call = lambda: hk.paged_decode_attn(q, Kp if n_kv else None, Vp if n_kv else None, Ap if n_act else None, tb, sl, bt, lp,
                                        n_act_used=n_act, out=out, absorbed=args.absorbed, cu_tokens=cu, total_tokens=total,
                                        workspace=ws)
    for _ in range(2):
        call()
    torch.cuda.synchronize()
    if args.graph:                                             # the step replayed from a HIP graph (nothing is allocated inside)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            hk.paged_decode_attn(q, Kp if n_kv else None, Vp if n_kv else None, Ap if n_act else None, tb, sl, bt, lp,
                                 n_act_used=n_act, out=out, absorbed=args.absorbed, cu_tokens=cu, total_tokens=total,
                                 workspace=ws, stream=torch.cuda.current_stream())
        call = graph.replay
        call()
    ts = []
    for _ in range(args.iters):
        e0, e1 = _events(torch)
        e0.record(); call(); e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ms = float(np.mean(ts))
    tokens = int(lens.sum())
    attn_bytes = float(tokens) * 4 * d                          # every token's K and V row once
    regen_flop = 4.0 * n_act * bt * d * d
    print(json.dumps({"entry": "hk_paged_decode_attn_absorbed" if args.absorbed else "hk_paged_decode_attn",
                      "workload": "%s: B=%d H=%d dh=%d L%s%d, %d-token blocks, %.0f %% ACT blocks" %
                                  (cfg.name, B, H, dh, "<=" if args.ragged else "=", L, bt, 100 * args.act_fraction),
                      "iters": args.iters, "replayed_from_graph": bool(args.graph), "ms": ms, "min_ms": float(np.min(ts)), "tokens": tokens, "act_blocks": n_act,
                      "kv_blocks": n_kv, "attention_bytes": attn_bytes, "regen_flop": regen_flop,
                      "attention_GBps_if_all_time_were_attention": attn_bytes / (ms * 1e-3) / 1e9}))
    return 0


def measure_loop(args):
    import ctypes
    import torch
    from . import binding as hk, synth
    cfg = synth.CONFIGS[args.config]
    B, d, H, dh, L, bt = cfg.B, cfg.d, cfg.n_heads, cfg.head_dim, cfg.L, args.block_tokens
    f16 = torch.float16
    rng = np.random.default_rng(cfg.seed)
    room = args.iters + 8                                      # tokens every request will take during the run
    lens = (rng.integers(L // 2, L + 1 - room, B) if args.ragged else np.full(B, L - room)).astype(np.int32)
    nb = (lens + bt - 1) // bt
    max_blocks = int((lens.max() + room + bt - 1) // bt)
    kinds = [rng.random(n) < args.act_fraction for n in nb]
    n_act = int(sum(int(k.sum()) for k in kinds)); n_kv = int(nb.sum()) - n_act
    spare = B * ((room + bt - 1) // bt + 1)
    P_kv, P_act = n_kv + spare, n_act + spare
    table = np.full((B, max_blocks), 0x7fffffff, np.int32)
    pa, pk = rng.permutation(max(n_act, 1)), rng.permutation(max(n_kv, 1))
    ia = ik = 0
    for b in range(B):
        for i in range(nb[b]):
            if kinds[b][i]:
                table[b, i] = ~int(pa[ia]); ia += 1
            else:
                table[b, i] = int(pk[ik]); ik += 1
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen, device="cuda") * std + mean).to(f16)
    kv_std = 0.02 * d ** 0.5
    Kp = torch.empty(P_kv, H, bt, dh, device="cuda", dtype=f16)
    Vp = torch.empty_like(Kp)
    step = max(1, (1 << 28) // (H * bt * dh))
    for i in range(0, P_kv, step):
        Kp[i:i + step] = rn(*Kp[i:i + step].shape, std=kv_std)
        Vp[i:i + step] = rn(*Vp[i:i + step].shape, std=kv_std)
    Ap = rn(P_act, bt, d)
    x = rn(B, d)
    Wq, bq = rn(d, d, std=0.02), rn(d, std=0.01)
    Wkv, bkv = rn(2 * d, d, std=0.02), rn(2 * d, std=0.01)
    ln_w, ln_b = rn(d, std=0.02, mean=1.0), rn(d, std=0.02)
    lp = (ln_w, ln_b, Wkv, bkv)
    lp = lp + (hk.prepare_layer(*lp, H),)
    tb, sl = torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda()
    cn = torch.tensor([n_kv, n_act, 0, 0], dtype=torch.int32, device="cuda")
    cu = torch.zeros(B + 1, dtype=torch.int64, device="cuda")
    q = torch.empty(B, H, dh, device="cuda", dtype=f16)
    out = torch.empty_like(q)
    bound = int(lens.sum()) + B * room                          # an upper bound of the tokens during the run
    shape = hk.make_shape(d, H)
    cache = hk.make_paged_cache(Kp, Vp, Ap, tb, sl, cu, bound, bt, P_act)
    ws_q = hk.new_workspace(hk.hk_qkv_workspace_bytes(shape, B))
    ws_a = hk.new_workspace(int(hk.lib().hk_paged_absorbed_workspace_bytes(ctypes.byref(shape), B, ctypes.byref(cache))))
    act_host, kv_host = max(1, round(100 * args.act_fraction)), max(0, 100 - round(100 * args.act_fraction))

    grew = torch.zeros(B, dtype=torch.int32, device="cuda")

    def one_step(stream):
        hk.paged_append(tb, sl, cu, cn, P_kv, P_act, bt, act_host, kv_host, stream=stream, grew=grew)
        hk.qkv_current_paged(x, *lp[:4], Wq, bq, H, Kp, Vp, Ap, tb, sl, bt, q_out=q, workspace=ws_q, stream=stream,
                             store_mask=grew)
        hk.paged_decode_attn(q, Kp, Vp, Ap, tb, sl, bt, lp, n_act_used=P_act, out=out, absorbed=True, cu_tokens=cu,
                             total_tokens=bound, workspace=ws_a, stream=stream)

    for _ in range(2):
        one_step(None)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step(torch.cuda.current_stream())
    graph.replay()
    ts = []
    for _ in range(args.iters):
        e0, e1 = _events(torch)
        e0.record(); graph.replay(); e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ms = float(np.mean(ts))
    stuck = int(cn[2].item())
    print(json.dumps({"entry": "hk_paged_append + hk_qkv_current_paged + hk_paged_decode_attn_absorbed, one HIP graph",
                      "workload": "%s: B=%d H=%d dh=%d L%s%d, %d-token blocks, %.0f %% ACT blocks" %
                                  (cfg.name, B, H, dh, "<=" if args.ragged else "=", L, bt, 100 * args.act_fraction),
                      "iters": args.iters, "ms": ms, "min_ms": float(np.min(ts)), "decode_tokens_per_s_per_layer": B / (ms * 1e-3),
                      "tokens_in_context_at_end": int(sl.sum().item()), "requests_that_could_not_grow": stuck}))
    return 0 if stuck == 0 else 1


def measure_overlap(args):
    import time
    import torch
    from . import binding as hk, synth
    from .hipevents import EventSet
    cfg = synth.CONFIGS[args.config]
    if cfg.L_kv == 0 or cfg.L_act == 0:
        cfg = cfg.with_ratio(0.5)                              # both segments are needed for anything to overlap
    B, d, H, dh = cfg.B, cfg.d, cfg.n_heads, cfg.head_dim
    f16 = torch.float16
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen, device="cuda") * std + mean).to(f16)
    kv_std = 0.02 * d ** 0.5
    lp = (rn(d, std=0.02, mean=1.0), rn(d, std=0.02), rn(2 * d, d, std=0.02), rn(2 * d, std=0.01))
    lp = lp + (hk.prepare_layer(*lp, H),)
    q = rn(B, H, dh, std=kv_std)
    act = torch.empty(B, cfg.L_act, d, device="cuda", dtype=f16)
    Kc = torch.empty(B, H, cfg.L_kv, dh, device="cuda", dtype=f16)
    Vc = torch.empty_like(Kc)
    for b in range(B):
        act[b] = rn(cfg.L_act, d)
        Kc[b] = rn(H, cfg.L_kv, dh, std=kv_std)
        Vc[b] = rn(H, cfg.L_kv, dh, std=kv_std)
    shape = hk.make_shape(d, H)
    out = torch.empty(B, H, dh, device="cuda", dtype=f16)
    ws1 = hk.new_workspace(hk.hk_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
    ws2 = hk.new_workspace(hk.hk_two_stream_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
    side = torch.cuda.Stream()
    ev = EventSet(2)
    cus = torch.cuda.get_device_properties(0).multi_processor_count

    def timed(call):
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.iters):
            call()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.iters * 1e3

    res = {"single_stream_entry_point_ms": timed(lambda: hk.hybrid_decode_attn(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws1)),
           "two_stream_call_on_one_stream_ms": timed(lambda: hk.hybrid_decode_attn_two_stream(q, Kc, Vc, act, lp, cfg.ratio, None, ev,
                                                                                               out=out, workspace=ws2))}
    for free in ((0, 8, 16, 32) if args.free_cus is None else (args.free_cus,)):
        res["two_streams_gemm_on_%d_cus_ms" % (cus - free)] = timed(
            lambda: hk.hybrid_decode_attn_two_stream(q, Kc, Vc, act, lp, cfg.ratio, side, ev, out=out, workspace=ws2,
                                                     gemm_cus=0 if free == 0 else cus - free))
    ev.destroy()
    print(json.dumps({"entry": "hk_hybrid_decode_attn_two_stream", "compute_units": cus,
                      "workload": "%s: B=%d d=%d H=%d L_kv=%d L_act=%d" % (cfg.name, B, d, H, cfg.L_kv, cfg.L_act),
                      "iters": args.iters, "result": res}))
    return 0


def measure_gemm(args):
    import torch
    from . import binding as hk, synth
    cfg = synth.CONFIGS[args.config]
    B, d, H, dh = cfg.B, cfg.d, cfg.n_heads, cfg.head_dim
    L = cfg.L_act if cfg.L_act else cfg.L
    f16 = torch.float16
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen, device="cuda") * std + mean).to(f16)
    act = torch.empty(B, L, d, device="cuda", dtype=f16)
    for b in range(B):
        act[b] = rn(L, d)
    W, bias = rn(2 * d, d, std=0.02), rn(2 * d, std=0.01)
    g, be = rn(d, std=0.02, mean=1.0), rn(d, std=0.02)
    K = torch.empty(B, H, L, dh, device="cuda", dtype=f16)
    V = torch.empty_like(K)
    shape = hk.make_shape(d, H)
    ws = hk.new_workspace(hk.hk_regen_workspace_bytes(shape, B, L))
    prep = hk.prepare_layer(g, be, W, bias, H)
    flop = 4.0 * B * L * d * d
    ours = lambda: hk.regen_kv(act, g, be, W, bias, H, K_out=K, V_out=V, workspace=ws, prepared=prep)
    a2 = act.view(B * L, d)
    out = torch.empty(B * L, 2 * d, device="cuda", dtype=f16)
    lib = lambda: torch.addmm(bias, a2, W.t(), out=out)

    def timed(f):
        e0, e1 = _events(torch)
        e0.record()
        for _ in range(args.iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.iters

    for _ in range(2):
        ours(); lib()
    rounds = []
    for _ in range(4):
        t1, t2 = timed(ours), timed(lib)
        rounds.append({"hk_regen_kv_tflops": flop / t1 / 1e9, "library_gemm_tflops": flop / t2 / 1e9})
    line = {"entry": "hk_regen_kv against torch.addmm (hipBLASLt), alternating, %d launches per figure" % args.iters,
            "workload": "%s: M=%d K=%d N=%d" % (cfg.name, B * L, d, 2 * d), "peak_tflops": 2500.0, "rounds": rounds}
    if args.candidates > 0:
        # every kernel the library offers for the plain GEMM (no bias, no LayerNorm, row-major output), its own order
        from . import probe
        ms = probe.library_gemm_candidates(a2, W, out, args.candidates, iters=3)
        tf = [round(flop / t / 1e9) if t > 0 else None for t in ms]
        line["library_candidates_tflops"] = tf
        line["library_candidates_best_tflops"] = max(x for x in tf if x is not None)
        line["hk_regen_kv_tflops_after_candidates"] = flop / timed(ours) / 1e9
    print(json.dumps(line))
    return 0


def measure_read(args):
    """The read rate of the checkpoint rows of a workload by shape of one load instruction (probe.read_rate)."""
    import torch
    from . import probe, synth
    cfg = synth.CONFIGS[args.config]
    rows = cfg.B * (cfg.L_act if cfg.L_act else cfg.L) // 128 * 128
    row_bytes = cfg.d * 2 // 1024 * 1024
    # normally distributed fp16 values: with MFMAs in the loop the clock, and with it the rate, depends on the data
    buf = torch.randn(rows * row_bytes // 2, dtype=torch.float16, device="cuda").view(torch.uint8)
    table = []
    for nt in (False, True):
        for rpl in (8, 4, 2, 1):
            table.append({"rows_per_load": rpl, "bytes_per_row_per_load": 1024 // rpl, "nontemporal": nt,
                          "GBps": probe.read_rate(buf, rows, row_bytes, rpl, nt, iters=args.iters)})
    parts = []
    for flags, what in ((0, "stream alone, 5 steps of 4 loads in flight"), (1, "+ a workgroup barrier per step"),
                        (2, "+ 3 loads per thread and step from rows every workgroup shares (L2)"), (3, "+ barrier + shared loads"),
                        (4, "+ every piece through a private LDS block"), (5, "+ barrier + LDS"), (6, "+ shared loads + LDS"),
                        (7, "+ barrier + shared loads + LDS"), (15, "+ barrier + shared loads + LDS + 12 MFMAs per step"),
                        (23, "+ barrier + shared loads + LDS + MFMAs + the shared operand through an LDS tile")):
        parts.append({"what": what, "GBps": probe.read_rate(buf, rows, row_bytes, 100 + flags, False, iters=args.iters)})
    print(json.dumps({"entry": "probe.read_rate (20 loads of 16 bytes per lane in flight per wavefront, 32 rows per wavefront)",
                      "workload": "%s: %d rows x %d bytes = %.2f GB" % (cfg.name, rows, row_bytes, rows * row_bytes / 1e9),
                      "peak_GBps": 8000.0, "table": table, "stream_with_parts_of_a_streaming_mfma_kernel": parts}))
    return 0


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["qkv", "paged", "loop", "overlap", "gemm", "read"])
    ap.add_argument("--config", default=None)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--block-tokens", type=int, default=16)
    ap.add_argument("--act-fraction", type=float, default=0.0)
    ap.add_argument("--ragged", action="store_true")
    ap.add_argument("--absorbed", action="store_true", help="paged: the entry point that does not regenerate K/V")
    ap.add_argument("--graph", action="store_true", help="paged: time the step replayed from a HIP graph")
    ap.add_argument("--candidates", type=int, default=0,
                    help="gemm: also time up to this many kernels the vendor library offers for the shape (its heuristic's list)")
    ap.add_argument("--free-cus", type=int, default=None, help="overlap: only this carve-out (compute units left to the side stream)")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("measure: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    from . import binding as hk
    hk.lib()
    if args.what == "qkv":
        args.config = args.config or "opt6.7b"
        return measure_qkv(args)
    if args.what == "loop":
        args.config = args.config or "opt6.7b"
        return measure_loop(args)
    if args.what == "overlap":
        args.config = args.config or "opt6.7b"
        return measure_overlap(args)
    if args.what == "read":
        return measure_read(args)
    if args.what == "gemm":
        args.config = args.config or "opt66b"
        if args.iters == 20:
            args.iters = 6
        return measure_gemm(args)
    args.config = args.config or "opt66b"
    return measure_paged(args)


if __name__ == "__main__":
    sys.exit(main())
