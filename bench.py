#!/usr/bin/env python3
"""Benchmark of the per-layer hybrid-cache decode step on one MI355X.

A step is one pass of the whole hot path (LayerNorm statistics -> K/V regeneration GEMM ->
single-query attention over cached ++ regenerated K/V -> merge) over one synthetic batch of the
OPT-6.7B-shaped workload (d=4096, 32 heads x 128, B=32, context 1024 at ratio 0.5), through the
C ABI.  Inputs are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config opt6.7b] [--no-cpu-baseline]
    python bench.py --sweep [--config opt66b]      ratio sweep (KV fraction 0 .. 1) with the balance point
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks used for the roofline fractions
PEAK_MFMA_F16_TFLOPS = 2500.0     # dense fp16 matrix, 256 CUs
PEAK_HBM_GBPS = 8000.0


def algorithmic_counts(cfg):
    """Algorithmic work of one step: regeneration GEMM flops (2*M*d*2d) and the bytes the
    attention must stream (K and V of every context token once: B*L*4d in fp16)."""
    gemm_flops = 4.0 * cfg.M * cfg.d * cfg.d
    attn_bytes = float(cfg.B) * cfg.L * 4 * cfg.d
    return gemm_flops, attn_bytes


def profiled_traffic(cfg_name):
    """HBM-side bytes per launch from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE / WRITE_SIZE, scaled against a plain copy of known size), or {} if there is none."""
    path = os.path.join(ROOT, "profiles", "hybrid_step_%s.txt" % cfg_name)
    out = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("TRAFFIC "):
                    parts = line.split()
                    kv = dict(p.split("=") for p in parts[1:] if "=" in p)
                    out[parts[1]] = (float(kv["fetch_kib"]) + float(kv["write_kib"])) * 1024.0
    except OSError:
        pass
    return out


def cpu_baseline(cfg, budget_s=15.0):
    """The CPU oracle (fp32 build, as it stands) timed on a bounded sample of the same workload:
    whole sequences of the batch, as many as fit the time budget."""
    from oracle import hybridkv_oracle as oracle
    from paper_2501_01792_amd import synth
    oracle.build()

    def run(n):
        b = synth.make_batch(cfg, sequences=range(n))
        t0 = time.perf_counter()
        out, _, _ = oracle.hybrid_decode_attn(b["q"], b["K_cache"] if cfg.L_kv else None,
                                              b["V_cache"] if cfg.L_kv else None,
                                              b["act"] if cfg.L_act else None,
                                              b["ln_w"], b["ln_b"], b["Wkv"], b["bkv"], cfg.n_heads,
                                              precision="f32")
        return time.perf_counter() - t0, out

    t1, out = run(1)
    n = int(max(1, min(cfg.B, budget_s // max(t1, 1e-3))))
    if n > 1:
        t, out = run(n)
    else:
        t = t1
    unit_tokens = max(cfg.L_act, 1)
    return {
        "value": n * unit_tokens / t, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "fp32 oracle, whole step on %d of %d sequences of the same workload (%d checkpoint + %d cached "
                  "tokens each), %.1f s" % (n, cfg.B, cfg.L_act, cfg.L_kv, t),
    }, n, out


def sweep(args):
    """Ratio sweep of one workload (Sec. 4.3): per KV fraction r the time of regeneration
    (LayerNorm statistics + projection: the paper's T_kv_gen of the (1-r) B L checkpointed tokens)
    and of attention, the least-squares line T_kv_gen(n) = a n + b over the sweep (the paper fits
    the same line, Sec. 4.3), and the ratio r* at which
    T_kv_gen((1-r) n) = T_load_w + T_load_kv(r n) (Eq. 8-10) for stated host-link bandwidths.
    The link is modelled (bytes / bandwidth), not measured: there is no host offload on this path.
    Inputs are drawn on the GPU with the distributions of the benchmark recipe (timing only)."""
    import numpy as np
    import torch
    from paper_2501_01792_amd import binding as hk, synth
    from paper_2501_01792_amd.hipevents import EventSet
    torch.cuda.set_device(0)
    base = synth.CONFIGS[args.config]
    d, H, dh, B, L = base.d, base.n_heads, base.head_dim, base.B, base.L
    gen = torch.Generator(device="cuda").manual_seed(base.seed)
    rn = lambda *shape, std=1.0, mean=0.0: (torch.randn(*shape, generator=gen, device="cuda", dtype=torch.float32) * std + mean).half()
    kv_std = 0.02 * d ** 0.5
    Wkv, bkv = rn(2 * d, d, std=0.02), rn(2 * d, std=0.01)
    ln_w, ln_b = rn(d, std=0.02, mean=1.0), rn(d, std=0.02)
    lp = (ln_w, ln_b, Wkv, bkv)
    lp = lp + (hk.prepare_layer(*lp, H),)
    q = rn(B, H, dh, std=kv_std)
    act_full = torch.empty((B, L, d), dtype=torch.float16, device="cuda")
    for b in range(B):
        act_full[b] = rn(L, d)
    K_full = torch.empty((B, H, L, dh), dtype=torch.float16, device="cuda")
    V_full = torch.empty_like(K_full)
    for b in range(B):
        K_full[b] = rn(H, L, dh, std=kv_std)
        V_full[b] = rn(H, L, dh, std=kv_std)
    out = torch.empty((B, H, dh), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream()
    rows = []
    for r in synth.SWEEP_RATIOS:
        cfg = base.with_ratio(r)
        Kc = K_full[:, :, :cfg.L_kv].contiguous() if cfg.L_kv else None
        Vc = V_full[:, :, :cfg.L_kv].contiguous() if cfg.L_kv else None
        act = act_full[:, cfg.L_kv:].contiguous() if cfg.L_act else None
        shape = hk.make_shape(d, H)
        ws = hk.new_workspace(hk.hk_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
        for _ in range(args.warmup):
            hk.hybrid_decode_attn(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
        events = [EventSet(5) for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in events:
            hk.hybrid_decode_attn(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream, events=e)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        dur = [float(np.mean([e.elapsed_ms(i, i + 1) for e in events])) for i in range(4)]
        for e in events:
            e.destroy()
        del ws
        ws = hk.new_workspace(hk.hk_absorbed_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
        for _ in range(2):
            hk.hybrid_decode_attn_absorbed(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            hk.hybrid_decode_attn_absorbed(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
        torch.cuda.synchronize()
        ms_absorbed = (time.perf_counter() - t0) / args.steps * 1e3
        rows.append({"ratio": r, "L_kv": cfg.L_kv, "L_act": cfg.L_act, "regen_tokens": cfg.M, "ms_per_step": ms,
                     "absorbed_ms_per_step": ms_absorbed,
                     "t_kv_gen_ms": dur[0] + dur[1], "t_attn_ms": dur[2] + dur[3],
                     "gemm_tflops": (4.0 * cfg.M * d * d / (dur[1] * 1e-3) / 1e12) if cfg.M else None,
                     "attn_gbps": float(B) * L * 4 * d / (dur[2] * 1e-3) / 1e9})
        del Kc, Vc, act, ws
        torch.cuda.empty_cache()
    n = np.array([x["regen_tokens"] for x in rows if x["regen_tokens"]], dtype=np.float64)
    t = np.array([x["t_kv_gen_ms"] for x in rows if x["regen_tokens"]], dtype=np.float64)
    a, b0, r2 = hk.fit_line(n, t)                                 # the library's least-squares line (Sec. 4.3)
    n_tot = float(B) * L
    balance = {}
    for name, gbps in (("pcie4_x16_32GBps (the paper's link)", 32.0), ("pcie5_x16_64GBps", 64.0)):
        per_tok_ms = 4.0 * d / (gbps * 1e9) * 1e3                  # T_load_kv per token of one layer (4d bytes, fp16)
        t_w_ms = 24.0 * d * d / (gbps * 1e9) * 1e3                 # T_load_w: 12 d^2 fp16 parameters of one decoder layer
        # a (1 - r) n + b = t_w + r n per_tok   ->   r = (a n + b - t_w) / (n (a + per_tok))
        r_star = (a * n_tot + b0 - t_w_ms) / (n_tot * (a + per_tok_ms))
        balance[name] = {"t_load_kv_ms_per_token": per_tok_ms, "t_load_w_ms": t_w_ms,
                         "kv_fraction_at_balance": float(min(1.0, max(0.0, r_star)))}
    print(json.dumps({"workload": "%s: d=%d H=%d B=%d L=%d" % (base.name, d, H, B, L), "steps": args.steps,
                      "sweep": rows, "t_kv_gen_fit": {"ms_per_token": float(a), "ms_offset": float(b0), "r2": r2},
                      "balance_model": balance}))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default=None)
    ap.add_argument("--ratio", type=float, default=None, help="override the KV fraction of the context")
    ap.add_argument("--gemm-tile", type=int, default=0)
    ap.add_argument("--attn-splits", type=int, default=0)
    ap.add_argument("--dtype", choices=["f16", "bf16"], default="f16",
                    help="bf16: the same step on bf16-rounded inputs (comparison; no CPU sample, no variants)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (the library allocates nothing and never synchronises, "
                         "so a caller can capture it); reported as graph_replay_ms_per_step, not as the benchmark's value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true", help="skip the comparison variants timed after the bench line's region")
    ap.add_argument("--absorbed", action="store_true",
                    help="time the comparison variant that does not regenerate K/V (hk_hybrid_decode_attn_absorbed) as the step; "
                         "prints its own line, not the benchmark's")
    ap.add_argument("--unprepared", action="store_true",
                    help="do not call hk_prepare_layer: the library prepares the layer inside every step")
    ap.add_argument("--sweep", action="store_true", help="ratio sweep of --config (default opt66b) instead of the bench line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of 1 GiB (3 launches) so that profiler byte counters "
                         "can be scaled against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step has no cross-GPU part); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2501_01792_amd import binding as hk, synth
    from paper_2501_01792_amd.hipevents import EventSet

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    hk.lib()
    if args.sweep:
        args.config = args.config or "opt66b"
        if args.steps == 50:
            args.steps, args.warmup = 5, 2
        return sweep(args)
    args.config = args.config or "opt6.7b"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    if args.ratio is not None:
        cfg = cfg.with_ratio(args.ratio)

    batch = synth.make_batch(cfg, threads=16)
    g = {k: torch.from_numpy(v).cuda() for k, v in batch.items()}
    if args.dtype == "bf16":
        g = {k: v.to(torch.bfloat16) for k, v in g.items()}
        args.no_cpu_baseline = args.no_variants = True
    lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
    prepare_ms = None
    if not args.unprepared and cfg.L_act:
        # One-time preparation of the layer (depends on its parameters only, not on the batch):
        # outside the timed region, like any weight pre-packing; its cost is reported.
        hk.prepare_layer(*lp, cfg.n_heads)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prepared = hk.prepare_layer(*lp, cfg.n_heads)
        torch.cuda.synchronize()
        prepare_ms = (time.perf_counter() - t0) * 1e3
        lp = lp + (prepared,)
    Kc = g["K_cache"] if cfg.L_kv else None
    Vc = g["V_cache"] if cfg.L_kv else None
    act = g["act"] if cfg.L_act else None
    shape = hk.make_shape(cfg.d, cfg.n_heads, attn_splits=args.attn_splits, gemm_tile=args.gemm_tile,
                          dtype=hk.HK_DTYPE_BF16 if args.dtype == "bf16" else hk.HK_DTYPE_F16)
    ws = hk.new_workspace(hk.hk_workspace_bytes(shape, cfg.B, cfg.L_kv, cfg.L_act))
    out = torch.empty((cfg.B, cfg.n_heads, cfg.head_dim), dtype=g["q"].dtype, device="cuda")
    stream = torch.cuda.current_stream()

    def step(events=None):
        hk.hybrid_decode_attn(g["q"], Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream,
                              attn_splits=args.attn_splits, gemm_tile=args.gemm_tile, events=events)

    if args.absorbed:
        del ws
        ws = hk.new_workspace(hk.hk_absorbed_workspace_bytes(shape, cfg.B, cfg.L_kv, cfg.L_act))

        def step(events=None):
            hk.hybrid_decode_attn_absorbed(g["q"], Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream,
                                           attn_splits=args.attn_splits)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    events = [EventSet(5) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    if args.absorbed:
        for e in events:
            e.destroy()
        ms = elapsed / args.steps * 1e3
        # bytes the variant has to move: the checkpoints twice, the cached K/V once, the prepared weights once
        nbytes = 2.0 * cfg.M * cfg.d * 2 + float(cfg.B) * cfg.L_kv * 4 * cfg.d + (4.0 * cfg.d * cfg.d if cfg.M else 0.0)
        line = {"metric": "absorbed_decode_context_tokens_per_s", "value": cfg.B * cfg.L / (ms * 1e-3), "unit": "tokens/s",
                "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
                "config": {"workload": "%s: d=%d H=%d B=%d L=%d ratio=%g, decode step of one layer without regenerating K/V "
                                       "(comparison variant)" % (cfg.name, cfg.d, cfg.n_heads, cfg.B, cfg.L, cfg.ratio)},
                "roofline": {"kernel": "whole step (all kernels)", "bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9,
                             "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                             "traffic": None}}
        if not args.no_cpu_baseline:
            base, n, ref = cpu_baseline(cfg)
            line["cpu_baseline"] = base
            got = out[:n].float().cpu().numpy()
            line["parity_vs_cpu_sample"] = {"max_abs": float(np.abs(got - ref).max()),
                                            "rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
        print(json.dumps(line))
        return 0

    # per-kernel durations from the events recorded on the launch stream inside the timed region
    names = ["ln_stats", "kv_gemm", "flash_decode", "merge_partials"]
    dur = {n: float(np.mean([e.elapsed_ms(i, i + 1) for e in events])) for i, n in enumerate(names)}
    for e in events:
        e.destroy()

    ms_per_step = elapsed / args.steps * 1e3
    gemm_flops, attn_bytes = algorithmic_counts(cfg)
    traffic = profiled_traffic(cfg.name) if args.ratio is None else {}
    gemm_kernel = "kv_gemm_fold_kernel"
    roofline = None
    if cfg.M > 0 and dur["kv_gemm"] > 0:
        ach = gemm_flops / (dur["kv_gemm"] * 1e-3) / 1e12
        roofline = {"kernel": "kv_gemm", "bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_F16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_F16_TFLOPS, "traffic": traffic.get(gemm_kernel),
                    "avg_ms": dur["kv_gemm"]}
    ach_bw = attn_bytes / (dur["flash_decode"] * 1e-3) / 1e9
    roofline_attn = {"kernel": "flash_decode", "bound": "hbm", "achieved": ach_bw, "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": ach_bw / PEAK_HBM_GBPS, "traffic": traffic.get("flash_decode_kernel"),
                     "avg_ms": dur["flash_decode"]}
    if roofline is None:
        roofline = roofline_attn

    result = {
        "metric": "regenerated_kv_tokens_per_s",
        "value": cfg.M / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "%s: d=%d H=%d dh=%d B=%d L=%d ratio=%g (L_kv=%d, L_act=%d), hybrid-cache decode step "
                               "of one layer" % (cfg.name, cfg.d, cfg.n_heads, cfg.head_dim, cfg.B, cfg.L, cfg.ratio,
                                                 cfg.L_kv, cfg.L_act),
                   "regen_gemm": "M=%d K=%d N=%d" % (cfg.M, cfg.d, 2 * cfg.d)},
        "decode_layer_latency_ms": ms_per_step,
        "decode_tokens_per_s": cfg.B / (ms_per_step * 1e-3),
        "regen_only_tokens_per_s": (cfg.M / ((dur["ln_stats"] + dur["kv_gemm"]) * 1e-3)) if cfg.M else None,
        "kernel_ms": dur,
        "layer_prepared": not args.unprepared,
        "prepare_layer_ms_once_per_layer": prepare_ms,
        "roofline": roofline,
        "roofline_attn": roofline_attn,
    }

    # What a loop of nothing but fp16 MFMAs sustains on this GPU: with random operands the shader
    # clock drops, so that rate (not the published peak) is the practical ceiling of the GEMM.
    from paper_2501_01792_amd import probe
    result["mfma_rate_probe_tflops"] = {"zero_operands": probe.mfma_rate(False), "random_operands": probe.mfma_rate(True)}
    if roofline.get("bound") == "mfma":
        roofline["frac_of_probe_random"] = roofline["achieved"] / result["mfma_rate_probe_tflops"]["random_operands"]

    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):                           # kernel attributes are set on first use: warm up before capture
            hk.hybrid_decode_attn(g["q"], Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=side,
                                  attn_splits=args.attn_splits, gemm_tile=args.gemm_tile)
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            hk.hybrid_decode_attn(g["q"], Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=torch.cuda.current_stream(),
                                  attn_splits=args.attn_splits, gemm_tile=args.gemm_tile)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["graph_replay_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3

    if not args.no_variants:
        # Comparison point beyond the paper (not part of `value`): the same step without regenerating K/V,
        # the projections moved to the query and to the weighted row sum (hk_hybrid_decode_attn_absorbed).
        ref_out = out.clone()
        ws2 = hk.new_workspace(hk.hk_absorbed_workspace_bytes(shape, cfg.B, cfg.L_kv, cfg.L_act))
        out2 = torch.empty_like(out)
        run2 = lambda: hk.hybrid_decode_attn_absorbed(g["q"], Kc, Vc, act, lp, cfg.ratio, out=out2, workspace=ws2,
                                                      stream=stream, attn_splits=args.attn_splits)
        for _ in range(3):
            run2()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run2()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) / args.steps * 1e3
        diff = (out2.float() - ref_out.float())
        result["absorbed_variant"] = {"ms_per_step": ms2, "speedup_vs_regenerating": ms_per_step / ms2,
                                      "max_abs_vs_regenerating": float(diff.abs().max()),
                                      "rel_l2_vs_regenerating": float(diff.norm() / ref_out.float().norm())}
        del ws2

    if not args.no_cpu_baseline:
        base, n, ref = cpu_baseline(cfg)
        result["cpu_baseline"] = base
        got = out[:n].float().cpu().numpy()
        result["parity_vs_cpu_sample"] = {"max_abs": float(np.abs(got - ref).max()),
                                          "rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
