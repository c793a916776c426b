"""Builds libsarathi.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsarathi.so")
SOURCES = ["api.cpp", "linear_api.cpp", "plan.cpp", "scheduler.cpp", "attn_kernels.hip", "linear_kernels.hip"]


def build_library(verbose: bool = False) -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature"
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(log + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libsarathi.so")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
