"""Writes the rocprofv3 summaries kept under profiles/: runs a benchmark command of this repository under
rocprofv3, one pass per counter group (kernel trace + stats; FETCH_SIZE; WRITE_SIZE; matrix-core counters; wait and
LDS counters; L2 hit / miss / fabric-read counters), and prints a short text summary of the per-kernel figures with
the commands that produced them.

    python3 -m paper_2501_01792_amd.profile_summary hybrid --config opt66b > profiles/hybrid_step_opt66b.txt
    python3 -m paper_2501_01792_amd.profile_summary hybrid --config opt66b --ratio 0.5 -- --absorbed > profiles/absorbed_step_...txt
    python3 -m paper_2501_01792_amd.profile_summary measure -- paged --config opt66b ... > profiles/paged_step_....txt

This process never touches the GPU: every pass is a child process `rocprofv3 ... -- python3 <program> ...` with a
time limit of its own, and a pass that fails ends the run.  Raw profiler output goes to a scratch folder beside the
sources (SCRATCH below), one sub-folder per program and pass; only the printed summary is meant to be kept.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SCRATCH = os.path.join("gpurun_out", "prof")      # raw profiler output, relative to ROOT

KERNELS = ("column_product|paged_scores|paged_index|paged_prefix|paged_append|row_stats|absorbed_scores_block|"
           "absorbed_scores|absorbed_softmax|absorbed_project_block|absorbed_project|absorbed_join|absorbed_stream|"
           "qkv_block|qkv_fused|ln_rows|qkv_finish|paged_decode|paged_merge|kv_gemm_fold|kv_gemm|prepare_layer|"
           "flash_decode|merge_partials|segment_join|mfma_rate|ln_stats[a-z_]*")

# counter groups, each within what one pass can hold (8 SQ, 4 TCC, 2 GRBM)
GROUPS = [
    ("mfma", ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_F16", "GRBM_GUI_ACTIVE"]),
    ("wait", ["SQ_WAVE_CYCLES", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY", "SQ_INSTS_LDS", "SQ_LDS_BANK_CONFLICT",
              "SQ_ACTIVE_INST_LDS", "SQ_INSTS_VALU", "SQ_WAVES"]),
    ("l2", ["TCC_HIT_sum", "TCC_MISS_sum", "TCC_EA0_RDREQ_sum", "TCC_EA0_RDREQ_DRAM_sum"]),
]


CALIBRATION = "device copy (runtime)"         # the runtime's buffer-copy kernel (tensor copies of the measured program); in
                                              # hybrid mode the program also makes one 1 GiB copy, its largest dispatch, which
                                              # calibrates the traffic counters


def short(name):
    m = re.search(r"(%s)_kernel(?:<|ILi)?(\d+)?" % KERNELS, name)
    if not m:
        if "Cijk_" in name:                                # a kernel of the vendor GEMM library (comparator runs)
            mt = re.search(r"MT(\d+x\d+x\d+)", name)
            return "library_gemm_%s_kernel" % (mt.group(1) if mt else "")
        return CALIBRATION if "rocclr_copyBuffer" in name else None     # (only used when the program was asked for the 1 GiB copy)
    return m.group(1) + ("<%s>" % m.group(2) if m.group(2) else "") + "_kernel"


def run_pass(tag, name, prof_args, prog, limit):
    out_dir = os.path.join(ROOT, SCRATCH, tag, name)
    shutil.rmtree(out_dir, ignore_errors=True)
    os.makedirs(out_dir, exist_ok=True)
    cmd = ["rocprofv3"] + prof_args + ["--output-format", "csv", "-d", out_dir, "-o", "p", "--"] + prog
    shown = " ".join(cmd).replace(ROOT + "/", "")
    env = dict(os.environ, TMPDIR="/tmp")
    print("[profile_summary] %s" % shown, file=sys.stderr, flush=True)
    with open(os.path.join(out_dir, "log.txt"), "w") as log:
        r = subprocess.run(["timeout", "-s", "KILL", str(limit)] + cmd, cwd=ROOT, env=env, stdout=log, stderr=subprocess.STDOUT)
    if r.returncode != 0:
        tail = open(os.path.join(out_dir, "log.txt")).read()[-2000:]
        raise SystemExit("pass %s failed (exit %d); end of its log:\n%s" % (name, r.returncode, tail))
    return out_dir, shown


def read_stats(out_dir):
    path = glob.glob(os.path.join(out_dir, "**", "p_kernel_stats.csv"), recursive=True)[0]
    rows = []
    for r in csv.DictReader(open(path)):
        s = short(r["Name"])
        if s:
            rows.append((s, int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
                         float(r["Percentage"])))
    return rows


def read_counters(out_dir):
    """{kernel: {counter: mean over dispatches}} and {kernel: dispatches}."""
    path = glob.glob(os.path.join(out_dir, "**", "p_counter_collection.csv"), recursive=True)[0]
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        s = short(r["Kernel_Name"])
        if s:
            agg[s][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (max(v) if k == CALIBRATION else sum(v) / len(v)) for c, v in cs.items()} for k, cs in agg.items()}


def program_line(out_dir):
    lines = [l.strip() for l in open(os.path.join(out_dir, "log.txt")) if l.startswith("{")]
    return lines[-1] if lines else None


def measure_traffic(config, ratio=None, dtype="f16", limit=150):
    """HBM-side bytes per launch of the kernels of bench.py's step on `config`, measured now: two short runs of
    bench.py under `rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each scaled by what the same
    counter reads for the 1 GiB device copy that bench.py adds when asked.  Returns {kernel name without template
    argument and "_kernel": bytes}.  For a caller that has not touched the GPU itself (the runs are child processes).
    Raises SystemExit (a pass failed) or RuntimeError (no calibration copy in the counters)."""
    tag = "live_%s%s" % (config, "_r%s" % ratio if ratio is not None else "")
    prog = ["python3", "bench.py", "--config", config, "--steps", "2", "--warmup", "1", "--dtype", dtype, "--no-cpu-baseline",
            "--no-variants", "--no-sweep", "--traffic", "none", "--calibrate-copy"] + (["--ratio", str(ratio)] if ratio is not None else [])
    df, _ = run_pass(tag, "fetch", ["--pmc", "FETCH_SIZE"], prog, limit)
    dw, _ = run_pass(tag, "write", ["--pmc", "WRITE_SIZE"], prog, limit)
    f, w = read_counters(df), read_counters(dw)
    if CALIBRATION not in f or CALIBRATION not in w:
        raise RuntimeError("the calibration copy is missing from the counters")
    sf, sw = 1048576.0 / f[CALIBRATION]["FETCH_SIZE"], 1048576.0 / w[CALIBRATION]["WRITE_SIZE"]
    out = {}
    for k in f:
        if k != CALIBRATION:
            name = k.split("<")[0].replace("_kernel", "")
            out[name] = (f[k].get("FETCH_SIZE", 0.0) * sf + w.get(k, {}).get("WRITE_SIZE", 0.0) * sw) * 1024.0
    out["_scale_factors"] = (sf, sw)
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["hybrid", "measure"], help="hybrid: bench.py (the benchmark's step); measure: python3 -m "
                    "paper_2501_01792_amd.measure with the arguments after --")
    ap.add_argument("--config", default="opt66b")
    ap.add_argument("--ratio", default=None)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--limit", type=int, default=240, help="seconds per pass")
    ap.add_argument("--skip", default="", help="comma-separated counter groups to leave out (mfma, wait, l2, traffic)")
    ap.add_argument("--timeline", type=int, default=0, help="also list start and end (us, relative) of the last N kernel "
                    "dispatches of the trace with their streams: shows whether kernels of two streams ran side by side")
    ap.add_argument("--extra", action="append", default=[], metavar="NAME:C1,C2,...",
                    help="one more counter pass (at most 8 SQ, 4 TCC, 2 GRBM counters), listed like the built-in groups")
    args, rest = ap.parse_known_args()
    args.rest = [a for a in rest if a != "--"]                 # what follows belongs to the measured program
    skip = set(x for x in args.skip.split(",") if x)

    if args.what == "hybrid":
        tag = "hybrid_%s%s" % (args.config, "_r" + args.ratio if args.ratio else "")
        tag += re.sub(r"[^A-Za-z0-9.]+", "_", " ".join(args.rest)).rstrip("_")
        prog = ["python3", "bench.py", "--config", args.config, "--steps", str(args.steps), "--warmup", "2", "--no-cpu-baseline",
                "--no-variants", "--no-sweep", "--traffic", "profiles"] + (["--ratio", args.ratio] if args.ratio else []) + args.rest
        calib = ["--calibrate-copy"]
        title = "hybrid-cache decode step, workload %s%s%s" % (args.config, " at KV fraction " + args.ratio if args.ratio else "",
                                                              ", bench.py " + " ".join(args.rest) if args.rest else "")
    else:
        tag = "measure_" + re.sub(r"[^A-Za-z0-9.]+", "_", " ".join(args.rest)).strip("_")
        prog = ["python3", "-m", "paper_2501_01792_amd.measure"] + args.rest
        calib = []
        title = "python3 -m paper_2501_01792_amd.measure " + " ".join(args.rest)

    out = ["rocprofv3 summary -- %s, MI355X (gfx950)" % title,
           "written by: python3 -m paper_2501_01792_amd.profile_summary %s" % " ".join(sys.argv[1:]), ""]

    d, shown = run_pass(tag, "stats", ["--kernel-trace", "--stats"], prog, args.limit)
    stats = read_stats(d)
    out += ["Kernel durations", "  command: " + shown, "",
            "  %-34s %6s %12s %12s %12s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "pct")]
    out += ["  %-34s %6d %12.1f %12.1f %12.1f %7.2f" % r for r in stats]
    if args.timeline > 0:
        path = glob.glob(os.path.join(d, "**", "p_kernel_trace.csv"), recursive=True)[0]
        rows = [r for r in csv.DictReader(open(path)) if short(r["Kernel_Name"]) and short(r["Kernel_Name"]) != CALIBRATION]
        rows.sort(key=lambda r: int(r["Start_Timestamp"]))
        rows = rows[-args.timeline:]
        t0 = int(rows[0]["Start_Timestamp"])
        out += ["", "Timeline of the last %d dispatches (us from the first of them; a kernel that starts before the previous "
                "one ends runs beside it)" % len(rows),
                "  %-34s %10s %12s %12s %10s" % ("kernel", "stream", "start_us", "end_us", "dur_us")]
        for r in rows:
            s0, s1 = (int(r["Start_Timestamp"]) - t0) / 1e3, (int(r["End_Timestamp"]) - t0) / 1e3
            out.append("  %-34s %10s %12.1f %12.1f %10.1f" % (short(r["Kernel_Name"]), r.get("Stream_Id", r.get("Queue_Id", "?")), s0, s1, s1 - s0))
    avg_us = {r[0]: r[2] for r in stats}
    # counter groups are listed for the kernels that matter: at least 0.5 % of the kernel time, never the calibration copy
    listed = set(r[0] for r in stats if r[5] >= 0.5 and r[0] != CALIBRATION)
    line = program_line(d)

    traffic = {}
    if "traffic" not in skip:
        df, shown_f = run_pass(tag, "fetch", ["--pmc", "FETCH_SIZE"], prog + calib, args.limit)
        dw, shown_w = run_pass(tag, "write", ["--pmc", "WRITE_SIZE"], prog + calib, args.limit)
        f, w = read_counters(df), read_counters(dw)
        out += ["", "HBM-side traffic counters (per dispatch, KiB)", "  commands: " + shown_f, "            " + shown_w, ""]
        sf = sw = None
        cal = CALIBRATION
        if calib and cal in f and cal in w:
            sf, sw = 1048576.0 / f[cal]["FETCH_SIZE"], 1048576.0 / w[cal]["WRITE_SIZE"]
            out.append("  calibration: a plain 1 GiB device copy (1048576 KiB read, 1048576 KiB written) reads FETCH_SIZE=%.1f, "
                       "WRITE_SIZE=%.1f" % (f[cal]["FETCH_SIZE"], w[cal]["WRITE_SIZE"]))
            out.append("               -> scale factors %.3f (fetch), %.3f (write)" % (sf, sw))
        else:
            sf, sw = 2.0, 1.0
            out.append("  no calibration copy in this program: the factors of the hybrid_step summaries are used (2.000 fetch: the counter "
                       "counts 64-byte units where the tool assumes 32; 1.000 write)")
        out.append("  %-34s %14s %14s %14s %14s %12s" % ("kernel", "FETCH_SIZE", "scaled KiB", "WRITE_SIZE", "scaled KiB", "GB/s (r+w)"))
        for k in sorted(f):
            if k == cal:
                continue
            fv, wv = f[k].get("FETCH_SIZE", 0.0), w.get(k, {}).get("WRITE_SIZE", 0.0)
            traffic[k] = (fv * sf, wv * sw)
            rate = (fv * sf + wv * sw) * 1024.0 / (avg_us[k] * 1e-6) / 1e9 if k in avg_us else float("nan")
            out.append("  %-34s %14.1f %14.1f %14.1f %14.1f %12.0f" % (k, fv, fv * sf, wv, wv * sw, rate))

    extra = [(e.split(":")[0], e.split(":")[1].split(",")) for e in args.extra]
    for name, counters in GROUPS + extra:
        if name in skip:
            continue
        dg, shown_g = run_pass(tag, name, ["--pmc"] + counters, prog, args.limit)
        c = read_counters(dg)
        out += ["", "Counters '%s' (mean per dispatch)" % name, "  command: " + shown_g, ""]
        for k in sorted(c):
            if k not in listed:
                continue
            for cn in counters:
                if cn in c[k]:
                    out.append("  %-34s %-32s %18.0f" % (k, cn, c[k][cn]))
            v = c[k]
            if name == "mfma" and v.get("GRBM_GUI_ACTIVE") and k in avg_us:
                cyc = v["GRBM_GUI_ACTIVE"] / 8.0                   # the counter is summed over the 8 XCDs
                out.append("  %-34s shader clock = GRBM_GUI_ACTIVE / 8 / avg duration = %.2f GHz" % (k, cyc / (avg_us[k] * 1e3)))
                if v.get("SQ_VALU_MFMA_BUSY_CYCLES"):
                    out.append("  %-34s matrix-core busy = MFMA_BUSY_CYCLES / (cycles x 1024 SIMDs) = %.1f %%"
                               % (k, 100.0 * v["SQ_VALU_MFMA_BUSY_CYCLES"] / (cyc * 1024.0)))
                if v.get("SQ_INSTS_VALU_MFMA_MOPS_F16"):
                    out.append("  %-34s matrix flops = MOPS_F16 x 512 = %.4e" % (k, v["SQ_INSTS_VALU_MFMA_MOPS_F16"] * 512.0))
            if name == "wait" and v.get("SQ_WAVE_CYCLES"):
                wc = v["SQ_WAVE_CYCLES"]
                out.append("  %-34s of the wave cycles: waiting (any) %.1f %%, waiting on an instruction %.1f %%, LDS instruction active %.1f %%; "
                           "LDS bank-conflict cycles per LDS instruction %.3f"
                           % (k, 100 * v.get("SQ_WAIT_ANY", 0) / wc, 100 * v.get("SQ_WAIT_INST_ANY", 0) / wc,
                              100 * v.get("SQ_ACTIVE_INST_LDS", 0) / wc,
                              v.get("SQ_LDS_BANK_CONFLICT", 0) / max(v.get("SQ_INSTS_LDS", 0), 1)))
            if name == "l2" and v.get("TCC_HIT_sum") is not None and v.get("TCC_MISS_sum") is not None:
                tot = v["TCC_HIT_sum"] + v["TCC_MISS_sum"]
                out.append("  %-34s L2 hit rate %.1f %% of %.3e requests; reads leaving L2 for the fabric %.3e, of them to memory "
                           "(last-level cache or HBM) %.3e" % (k, 100 * v["TCC_HIT_sum"] / max(tot, 1), tot,
                                                               v.get("TCC_EA0_RDREQ_sum", 0), v.get("TCC_EA0_RDREQ_DRAM_sum", 0)))

    if line:
        import json
        try:
            j = json.loads(line)
            keep = {k: j[k] for k in ("metric", "value", "unit", "ms_per_step", "ms", "min_ms", "kernel_ms", "workload", "entry", "result") if k in j}
            if isinstance(j.get("config"), dict):
                keep["workload"] = j["config"].get("workload")
            for k in ("roofline", "roofline_attn"):
                if isinstance(j.get(k), dict):
                    keep[k] = {x: j[k][x] for x in ("kernel", "achieved", "unit", "frac", "avg_ms") if x in j[k]}
            line = json.dumps(keep)
        except ValueError:
            pass
        out += ["", "The program's own figures (stats pass):", line]
    if traffic:
        out += ["", "Machine-readable copy of the scaled traffic (read by bench.py for roofline.traffic):"]
        out += ["TRAFFIC %s fetch_kib=%.1f write_kib=%.1f" % (k, v[0], v[1]) for k, v in sorted(traffic.items())]
    print("\n".join(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
