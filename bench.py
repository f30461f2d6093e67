#!/usr/bin/env python3
"""Benchmark of the per-layer hybrid-cache decode step on one MI355X.

A step is one pass of the whole hot path (LayerNorm statistics -> K/V regeneration GEMM ->
single-query attention over cached ++ regenerated K/V -> merge) over one synthetic batch, through
the C ABI.  The default workload is the largest one of the benchmark contract that fits one GPU:
the OPT-66B-shaped layer (d=9216, 72 heads x 128, B=64, context 4096) with every context token
regenerated (KV fraction 0: the regeneration GEMM is M=262144, K=9216, N=18432).  Inputs are
resident in HBM before the timed region.  Prints one JSON line, which also carries the KV-fraction
sweep {0, .25, .5, .75, 1} of the same layer (Sec. 4.3: where recomputation and cache streaming
balance) and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config opt66b] [--ratio R]
                    [--no-sweep] [--no-cpu-baseline] [--no-variants] [--traffic auto|live|profiles|none]
    python bench.py --sweep [--config opt66b]      only the sweep, as its own JSON line
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
# the targets the benchmark contract sets for the two kernels (fractions of those peaks)
TARGET_MFMA_FRAC = 0.60
TARGET_HBM_FRAC = 0.70
LAST_LEVEL_CACHE_BYTES = 256 << 20


def algorithmic_counts(cfg):
    """Algorithmic work of one step: regeneration GEMM flops (2*M*d*2d) and the bytes the
    attention must stream (K and V of every context token once: B*L*4d in fp16)."""
    gemm_flops = 4.0 * cfg.M * cfg.d * cfg.d
    attn_bytes = float(cfg.B) * cfg.L * 4 * cfg.d
    return gemm_flops, attn_bytes


def profiled_traffic(cfg_name):
    """HBM-side bytes per launch from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE / WRITE_SIZE, scaled against a plain copy of known size; written by
    ``python -m paper_2501_01792_amd.profile_summary``), or {} if there is none."""
    path = os.path.join(ROOT, "profiles", "hybrid_step_%s.txt" % cfg_name)
    out = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("TRAFFIC "):
                    parts = line.split()
                    kv = dict(p.split("=") for p in parts[1:] if "=" in p)
                    name = parts[1].split("<")[0].replace("_kernel", "")      # "kv_gemm_fold<4>_kernel" -> "kv_gemm_fold"
                    out[name] = (float(kv["fetch_kib"]) + float(kv["write_kib"])) * 1024.0
    except OSError:
        pass
    return out


def cpu_baseline(cfg, budget_s=15.0):
    """The CPU oracle (fp32 build, as it stands) timed on a bounded sample of the same workload:
    whole sequences of the batch, as many as fit the time budget (at least one)."""
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


def ratio_sweep(base, act_full, lp, q, steps, warmup, with_absorbed=True):
    """KV-fraction sweep of one layer (Sec. 4.3): per fraction r the time of regeneration (LayerNorm
    statistics + projection: the paper's T_kv_gen of the (1-r) B L checkpointed tokens) and of attention with
    their roofline fractions, the least-squares line T_kv_gen(n) = a n + b over the sweep (the paper fits the
    same line, Sec. 4.3; the library's hk_fit_line), and the fraction r* at which
    T_kv_gen((1-r) n) = T_load_w + T_load_kv(r n) (Eq. 8-10) for stated host-link bandwidths.  The link is
    modelled (bytes / bandwidth), not measured: there is no host offload on this path.
    ``act_full [B, L, d]`` are the layer inputs of every context token (the checkpoints of fraction r are its
    last (1-r) L tokens); the cached K/V rows are drawn here on the GPU with the recipe's moments (the step is
    defined for any cache content; timing only)."""
    import numpy as np
    import torch
    from paper_2501_01792_amd import binding as hk, synth
    from paper_2501_01792_amd.hipevents import EventSet
    d, H, dh, B, L = base.d, base.n_heads, base.head_dim, base.B, base.L
    gen = torch.Generator(device="cuda").manual_seed(base.seed)
    kv_std = 0.02 * d ** 0.5
    K_full = torch.empty((B, H, L, dh), dtype=torch.float16, device="cuda")
    V_full = torch.empty_like(K_full)
    for b in range(B):
        K_full[b] = (torch.randn(H, L, dh, generator=gen, device="cuda") * kv_std).half()
        V_full[b] = (torch.randn(H, L, dh, generator=gen, device="cuda") * kv_std).half()
    out = torch.empty((B, H, dh), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream()
    shape = hk.make_shape(d, H)
    rows = []
    for r in synth.SWEEP_RATIOS:
        cfg = base.with_ratio(r)
        Kc = K_full[:, :, :cfg.L_kv].contiguous() if cfg.L_kv else None
        Vc = V_full[:, :, :cfg.L_kv].contiguous() if cfg.L_kv else None
        act = (act_full if cfg.L_kv == 0 else act_full[:, cfg.L_kv:].contiguous()) if cfg.L_act else None
        ws = hk.new_workspace(hk.hk_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
        for _ in range(warmup):
            hk.hybrid_decode_attn(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
        events = [EventSet(5) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in events:
            hk.hybrid_decode_attn(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream, events=e)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        dur = [float(np.mean([e.elapsed_ms(i, i + 1) for e in events])) for i in range(4)]
        for e in events:
            e.destroy()
        del ws
        row = {"ratio": r, "L_kv": cfg.L_kv, "L_act": cfg.L_act, "regen_tokens": cfg.M, "ms_per_step": ms,
               "t_kv_gen_ms": dur[0] + dur[1], "t_attn_ms": dur[2] + dur[3],
               "gemm_tflops": None, "gemm_frac_of_mfma_peak": None,
               "attn_gbps": float(B) * L * 4 * d / (dur[2] * 1e-3) / 1e9}
        row["attn_frac_of_hbm_peak"] = row["attn_gbps"] / PEAK_HBM_GBPS
        if cfg.M:
            row["gemm_tflops"] = 4.0 * cfg.M * d * d / (dur[1] * 1e-3) / 1e12
            row["gemm_frac_of_mfma_peak"] = row["gemm_tflops"] / PEAK_MFMA_F16_TFLOPS
        if with_absorbed:
            ws = hk.new_workspace(hk.hk_absorbed_workspace_bytes(shape, B, cfg.L_kv, cfg.L_act))
            for _ in range(2):
                hk.hybrid_decode_attn_absorbed(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                hk.hybrid_decode_attn_absorbed(q, Kc, Vc, act, lp, cfg.ratio, out=out, workspace=ws, stream=stream)
            torch.cuda.synchronize()
            row["absorbed_ms_per_step"] = (time.perf_counter() - t0) / steps * 1e3
            del ws
        rows.append(row)
        del Kc, Vc, act
        torch.cuda.empty_cache()
    n = np.array([x["regen_tokens"] for x in rows if x["regen_tokens"]], dtype=np.float64)
    t = np.array([x["t_kv_gen_ms"] for x in rows if x["regen_tokens"]], dtype=np.float64)
    a, b0, r2 = hk.fit_line(n, t)                                 # the library's least-squares line (Sec. 4.3)
    n_tot = float(B) * L
    per_tok_hbm_ms = 4.0 * d / (PEAK_HBM_GBPS * 1e9) * 1e3
    balance = {"against_hbm_alone": {
        "t_stream_ms_per_cached_token_at_peak": per_tok_hbm_ms, "t_kv_gen_ms_per_token": float(a),
        "note": "regeneration costs %.0fx what streaming a cached token from HBM costs: inside one GPU the fastest "
                "split is all-KV; the balance of Sec. 4.3 is against the host link" % (a / per_tok_hbm_ms)}}
    for name, gbps in (("pcie4_x16_32GBps (the paper's link)", 32.0), ("pcie5_x16_64GBps", 64.0)):
        per_tok_ms = 4.0 * d / (gbps * 1e9) * 1e3                  # T_load_kv per token of one layer (4d bytes, fp16)
        t_w_ms = 24.0 * d * d / (gbps * 1e9) * 1e3                 # T_load_w: 12 d^2 fp16 parameters of one decoder layer
        # a (1 - r) n + b = t_w + r n per_tok   ->   r = (a n + b - t_w) / (n (a + per_tok))
        r_star = (a * n_tot + b0 - t_w_ms) / (n_tot * (a + per_tok_ms))
        balance[name] = {"t_load_kv_ms_per_token": per_tok_ms, "t_load_w_ms": t_w_ms, "modelled": True,
                         "kv_fraction_at_balance": float(min(1.0, max(0.0, r_star)))}
    del K_full, V_full
    torch.cuda.empty_cache()
    return {"workload": "%s: d=%d H=%d B=%d L=%d" % (base.name.split("@")[0], d, H, B, L), "steps": steps, "warmup": warmup,
            "rows": rows, "t_kv_gen_fit": {"ms_per_token": float(a), "ms_offset": float(b0), "r2": r2},
            "balance_model": balance}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="opt66b")
    ap.add_argument("--ratio", type=float, default=None, help="override the KV fraction of the context")
    ap.add_argument("--gemm-tile", type=int, default=0)
    ap.add_argument("--attn-splits", type=int, default=0)
    ap.add_argument("--dtype", choices=["f16", "bf16"], default="f16",
                    help="bf16: the same step on bf16-rounded inputs (comparison; no CPU sample, no variants, no sweep)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (the library allocates nothing and never synchronises, "
                         "so a caller can capture it); reported as graph_replay_ms_per_step, not as the benchmark's value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true", help="skip the comparison variants timed after the bench line's region")
    ap.add_argument("--no-sweep", action="store_true", help="skip the KV-fraction sweep that follows the timed region")
    ap.add_argument("--sweep-steps", type=int, default=5)
    ap.add_argument("--absorbed", action="store_true",
                    help="time the comparison variant that does not regenerate K/V (hk_hybrid_decode_attn_absorbed) as the step; "
                         "prints its own line, not the benchmark's")
    ap.add_argument("--unprepared", action="store_true",
                    help="do not call hk_prepare_layer: the library prepares the layer inside every step")
    ap.add_argument("--sweep", action="store_true", help="only the KV-fraction sweep of --config, as its own JSON line")
    ap.add_argument("--traffic", choices=["auto", "live", "profiles", "none"], default="auto",
                    help="where roofline.traffic (HBM-side bytes per launch) comes from: live = measured now, before this "
                         "process touches the GPU, by two short child runs of this program under rocprofv3 --pmc (FETCH_SIZE, "
                         "WRITE_SIZE, scaled by a 1 GiB copy); profiles = the committed summary of the workload; auto = live "
                         "for the benchmark's own line when rocprofv3 is there, else profiles")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of 1 GiB (3 launches) so that profiler byte counters "
                         "can be scaled against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step has no cross-GPU part); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        return 2

    # roofline.traffic measured in this run: child processes under the profiler, started before this process has
    # loaded anything that touches the GPU
    live_traffic, live_note = None, None
    main_line = not (args.sweep or args.absorbed or args.calibrate_copy)
    if args.traffic == "live" or (args.traffic == "auto" and main_line):
        import shutil
        if shutil.which("rocprofv3") is None:
            live_note = "rocprofv3 not found"
        else:
            try:
                from paper_2501_01792_amd import profile_summary
                live_traffic = profile_summary.measure_traffic(args.config, args.ratio, args.dtype)
            except (SystemExit, Exception) as e:                      # a failed pass must not cost the bench line
                live_note = "live measurement failed: %s" % (str(e).splitlines()[0] if str(e) else type(e).__name__)

    import numpy as np
    import torch
    from paper_2501_01792_amd import binding as hk, synth
    from paper_2501_01792_amd.hipevents import EventSet

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    hk.lib()
    torch.cuda.set_device(0)
    base = synth.CONFIGS[args.config]
    cfg = base if args.ratio is None else base.with_ratio(args.ratio)
    # the sweep needs the layer inputs of every context token: draw the batch with all tokens as checkpoints
    # (per-sequence streams: the checkpoints of a KV fraction r are the last (1-r) L tokens of the same draw)
    want_sweep = args.sweep or (not args.no_sweep and args.dtype == "f16" and not args.absorbed and args.ratio is None)
    full = base.with_ratio(0.0)

    if args.sweep:
        b = synth.make_batch(full, threads=16)
        g = {k: torch.from_numpy(v).cuda() for k, v in b.items()}
        lp = (g["ln_w"], g["ln_b"], g["Wkv"], g["bkv"])
        lp = lp + (hk.prepare_layer(*lp, base.n_heads),)
        res = ratio_sweep(base, g["act"], lp, g["q"], args.sweep_steps, 2)
        print(json.dumps(res))
        return 0

    batch = synth.make_batch(cfg, threads=16)
    g = {k: torch.from_numpy(v).cuda() for k, v in batch.items()}
    del batch
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
            cb, n, ref = cpu_baseline(cfg)
            line["cpu_baseline"] = cb
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
    if live_traffic:
        traffic = live_traffic
        traffic_source = ("measured in this run: two child runs of this program under rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE, "
                          "KiB per dispatch), scaled by what the same counters read for a 1 GiB device copy (factors %.3f and %.3f)"
                          % live_traffic["_scale_factors"])
    elif args.traffic == "none":
        traffic, traffic_source = {}, None
    else:
        traffic = profiled_traffic(cfg.name) if args.ratio is None else {}
        traffic_source = ("profiles/hybrid_step_%s.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE per launch, scaled by a 1 GiB copy)%s"
                          % (cfg.name, "; " + live_note if live_note else ""))
    gemm_kernel = "kv_gemm_fold"
    roofline = None
    if cfg.M > 0 and dur["kv_gemm"] > 0:
        ach = gemm_flops / (dur["kv_gemm"] * 1e-3) / 1e12
        roofline = {"kernel": "kv_gemm", "bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_F16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_F16_TFLOPS, "traffic": traffic.get(gemm_kernel),
                    "traffic_source": traffic_source if traffic.get(gemm_kernel) else None,
                    "algorithmic_flop": gemm_flops, "algorithmic_min_bytes": 6.0 * cfg.M * cfg.d + 4.0 * cfg.d * cfg.d,
                    "avg_ms": dur["kv_gemm"], "target_frac": TARGET_MFMA_FRAC,
                    "meets_target": ach / PEAK_MFMA_F16_TFLOPS >= TARGET_MFMA_FRAC}
    ach_bw = attn_bytes / (dur["flash_decode"] * 1e-3) / 1e9
    roofline_attn = {"kernel": "flash_decode", "bound": "hbm", "achieved": ach_bw, "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": ach_bw / PEAK_HBM_GBPS, "traffic": traffic.get("flash_decode"),
                     "algorithmic_bytes": attn_bytes, "avg_ms": dur["flash_decode"], "target_frac": TARGET_HBM_FRAC,
                     "meets_target": ach_bw / PEAK_HBM_GBPS >= TARGET_HBM_FRAC}
    if attn_bytes < 4 * LAST_LEVEL_CACHE_BYTES:
        roofline_attn["cache_assisted"] = ("the K/V stream of this workload (%.0f MB, part of it just written by the projection) is "
                                           "comparable to the 256 MB last-level cache: the rate is not a pure HBM rate"
                                           % (attn_bytes / 1e6))
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

    sample_out = out.clone()                                    # the step's output, before anything else reuses `out`
    del ws

    if not args.no_variants:
        # Comparison point beyond the paper (not part of `value`): the same step without regenerating K/V,
        # the projections moved to the query and to the weighted row sum (hk_hybrid_decode_attn_absorbed).
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
        diff = (out2.float() - sample_out.float())
        result["absorbed_variant"] = {"ms_per_step": ms2, "speedup_vs_regenerating": ms_per_step / ms2,
                                      "max_abs_vs_regenerating": float(diff.abs().max()),
                                      "rel_l2_vs_regenerating": float(diff.norm() / sample_out.float().norm())}
        del ws2

    if want_sweep:
        # The sweep of the same layer, after the timed region (it is not part of `value`).  With the bench
        # workload at KV fraction 0 its checkpoints are the layer inputs of every context token already.
        if cfg.L_kv == 0:
            act_full = act
        else:
            del act, Kc, Vc
            g.pop("act", None); g.pop("K_cache", None); g.pop("V_cache", None)
            torch.cuda.empty_cache()
            act_full = torch.from_numpy(synth.make_batch(full, threads=16)["act"]).cuda()
        result["ratio_sweep"] = ratio_sweep(base, act_full, lp, g["q"], args.sweep_steps, 2, with_absorbed=not args.no_variants)

    if not args.no_cpu_baseline:
        cb, n, ref = cpu_baseline(cfg)
        result["cpu_baseline"] = cb
        got = sample_out[:n].float().cpu().numpy()
        result["parity_vs_cpu_sample"] = {"max_abs": float(np.abs(got - ref).max()),
                                          "rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
