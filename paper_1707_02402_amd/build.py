"""Builds libdynbatch.so (HIP kernels + host planner + C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdynbatch.so")
SOURCES = ["planner.cpp", "timing.cpp", "iep_exec.hip", "iep_backward.hip", "moe.hip", "head.hip", "probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def build_library(verbose: bool = False, extra=()) -> str:
    """Compiles every source, every time it is called."""
    cmd = ["hipcc", *HIPCC_FLAGS, *extra, "-o", LIB]
    for s in sources():
        cmd += (["-x", "hip", s] if s.endswith(".hip") else ["-x", "hip", s])
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
