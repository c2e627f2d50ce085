"""Builds libtamoe.so (the C-ABI library of HIP kernels) in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtamoe.so")
# yardstick kernels that only bench.py calls: a library of their own, nothing shared with libtamoe.so
BENCH_CSRC = os.path.join(HERE, "csrc_bench")
BENCH_LIB = os.path.join(HERE, "libtamoe_bench.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # the compiler must not form packed fp32 instructions from ordinary float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]
OBJ_DIR = os.path.join(HERE, "_build")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def bench_sources():
    return sorted(glob.glob(os.path.join(BENCH_CSRC, "*.hip")))


def _headers():
    return (glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
            + glob.glob(os.path.join(BENCH_CSRC, "*.h")))


def _fresh(obj: str, src: str) -> bool:
    """True if obj is newer than its source and every header."""
    if not os.path.exists(obj):
        return False
    t = os.path.getmtime(obj)
    return all(os.path.getmtime(f) < t for f in [src, *_headers()])


def _compile(hipcc: str, src: str, verbose: bool, incremental: bool = False):
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
    if incremental and _fresh(obj, src):
        return obj, subprocess.CompletedProcess([], 0, "", "")
    # .cpp files hold host code only but share the HIP headers
    inc = ["-I", BENCH_CSRC] if os.path.dirname(src) == BENCH_CSRC else ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd = [hipcc, *HIPCC_FLAGS, *inc, "-x", "hip", "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    return obj, res


def build(verbose: bool = False, jobs: int = 0, incremental: bool = False) -> str:
    """Compiles every source of csrc/ to an object (in parallel: the gate's tile code is instantiated
    in one translation unit per element type) and links libtamoe.so.  incremental: keep the objects
    that are newer than their source and every header (for development; the default rebuilds all)."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources() + bench_sources()
    jobs = jobs or max(1, min(len(srcs), os.cpu_count() or 1, 8))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        done = list(pool.map(lambda src: _compile(hipcc, src, verbose, incremental), srcs))
    objs, bench_objs = [], []
    for src, (obj, res) in zip(srcs, done):
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed compiling {src}")
        if verbose and res.stderr.strip():
            sys.stderr.write(res.stderr)
        (bench_objs if os.path.dirname(src) == BENCH_CSRC else objs).append(obj)
    for out, parts in ((LIB, objs), (BENCH_LIB, bench_objs)):
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *parts, "-o", out]
        if verbose:
            print(" ".join(link), flush=True)
        res = subprocess.run(link, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed linking {out}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv[1:]))
