"""Build libukst.so (HIP, gfx950) in-tree with hipcc.  Run: python -m paper_2502_20493_amd.build"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libukst.so")
BENCH_LIB = os.path.join(HERE, "libukst_bench.so")  # measurement helpers, not part of the product

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept off on purpose (scalar fp32 code only)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
OBJDIR = os.path.join(HERE, "_build")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def bench_sources():
    return sorted(glob.glob(os.path.join(CSRC, "bench", "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    if verbose and out.strip():
        print(out)


def build_library(verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link libukst.so; csrc/bench/*.hip
    become libukst_bench.so (the benchmark's measured ceilings)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    srcs, bsrcs = sources(), bench_sources()
    objs = [os.path.join(OBJDIR, os.path.basename(s)[:-4] + ".o") for s in srcs]
    bobjs = [os.path.join(OBJDIR, "bench_" + os.path.basename(s)[:-4] + ".o") for s in bsrcs]
    jobs = jobs or max(1, min(len(srcs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1)), 16))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        futs = [pool.submit(_run, [hipcc] + HIPCC_FLAGS + ["-c", s, "-o", o], verbose)
                for s, o in zip(srcs + bsrcs, objs + bobjs)]
        for f in futs:
            f.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + bobjs + ["-o", BENCH_LIB], verbose)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(BENCH_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(BENCH_LIB))
    deps = sources() + bench_sources() + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
