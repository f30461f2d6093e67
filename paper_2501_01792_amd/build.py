"""Build libhybridkv.so (hand-written HIP for gfx950) in-tree with hipcc.

``python -m paper_2501_01792_amd.build`` compiles every source under csrc/ and links the
shared library next to this file.  No GPU is needed: hipcc cross-compiles.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhybridkv.so")
PROBE_SRC = [os.path.join(HERE, "probe", "mfma_rate.hip"),     # measurement aids: a library of their own
             os.path.join(HERE, "probe", "read_rate.hip")]
PROBE_LIB = os.path.join(HERE, "probe", "libhkprobe.so")
PROBE_LT_SRC = os.path.join(HERE, "probe", "library_gemm.hip")  # the vendor GEMM's candidate kernels, timed (links hipBLASLt)
PROBE_LT_LIB = os.path.join(HERE, "probe", "libhkprobe_lt.so")
SOURCES = ["api.hip", "device_info.hip", "ln_stats.hip", "kv_gemm.hip", "kv_gemm_fold.hip", "flash_decode.hip", "paged_decode.hip", "paged_append.hip", "qkv_current.hip", "absorbed.hip", "policy.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    tmp = PROBE_LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([HIPCC, *FLAGS, "-shared", *PROBE_SRC, "-o", tmp], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (PROBE_SRC, r.stdout, r.stderr))
    os.replace(tmp, PROBE_LIB)
    tmp = PROBE_LT_LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([HIPCC, *FLAGS, "-shared", PROBE_LT_SRC, "-o", tmp, "-lhipblaslt"], capture_output=True, text=True)
    if r.returncode != 0:
        # only `measure gemm --candidates` needs it: a toolchain without the vendor GEMM library still builds the rest
        print("build: %s not built (hipcc: %s)" % (PROBE_LT_LIB, (r.stderr.strip().splitlines() or ["?"])[-1]), file=sys.stderr)
    else:
        os.replace(tmp, PROBE_LT_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
