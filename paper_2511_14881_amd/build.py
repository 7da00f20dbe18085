"""Compiles the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU).  The
sources are compiled in parallel, one object per translation unit, and linked into one shared
library."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(CSRC, "libsilvertorch.so")
SOURCES = ["silvertorch.hip", "st_mfma_ks1.hip", "st_mfma_ks2.hip", "st_mfma_ks4.hip", "st_mfma_ks8.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed fp32 instructions stay off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra",
]


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    objs = [os.path.join(CSRC, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    jobs = [["hipcc", *HIPCC_FLAGS, *extra_flags, "-c", "-o", o, os.path.join(CSRC, s)] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1)) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], verbose)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
