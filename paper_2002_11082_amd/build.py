"""Builds libogq.so (HIP kernels + C ABI) for gfx950 with hipcc.  Run: python -m paper_2002_11082_amd.build

The library is compiled as several object files in parallel (the random-rounding kernels once per bucket
capacity) and linked into one shared library.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libogq.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    # the rounding test and the level arithmetic are specified one rounding per operation
    "-ffp-contract=off",
    # no packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]

# (source, extra flags, object name); the heaviest first so that they do not end up last in the pool
ROUNDING_PARTS = (16, 108, 104, 102, 8, 4, 2, 1)
UNITS = [("rounding_part.hip", [f"-DOGQ_PART={part}"], f"rounding_{part}.o") for part in ROUNDING_PARTS] + [
    ("bingrad.hip", [], "bingrad.o"),
    ("decode.hip", [], "decode.o"),
    ("api.hip", [], "api.o"),
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def build(verbose: bool = False, jobs: int = 0) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or max(1, min(len(UNITS), os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))
    shutil.rmtree(OBJ, ignore_errors=True)
    os.makedirs(OBJ)
    objects = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        futures = []
        for src, extra, obj in UNITS:
            out = os.path.join(OBJ, obj)
            objects.append(out)
            futures.append(pool.submit(_run, [hipcc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", out], verbose))
        for f in futures:
            f.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", LIB], verbose)
    shutil.rmtree(OBJ, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
