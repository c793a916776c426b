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


def build_sanitized_host(out_dir: str) -> str:
    """CPU-only build for AddressSanitizer + UndefinedBehaviorSanitizer: the host translation units of the library
    (validation, planner, scheduler, entry-point bookkeeping) against stand-ins for the HIP runtime and the kernel
    launchers, plus the fp64 checker's C sources, linked with the driver tests/sanitize/host_paths.cpp.
    Nothing of it runs on a GPU.  Returns the path of the executable."""
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", "/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"]
    objs = []
    for src in ("attention_oracle.c", "linear_oracle.c"):
        obj = os.path.join(out_dir, src + ".o")
        subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra"] + san + ["-c", os.path.join(ROOT, "oracle", src), "-o", obj], check=True)
        objs.append(obj)
    exe = os.path.join(out_dir, "host_paths_sanitized")
    cpp = [os.path.join(CSRC, s) for s in ("api.cpp", "plan.cpp", "scheduler.cpp")] + [os.path.join(ROOT, "tests", "sanitize", "host_paths.cpp")]
    res = subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Wno-unused-parameter", "-fopenmp", "-static-libasan"] + san + inc + cpp + objs +
                         ["-o", exe, "-lm"], capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("g++ failed building the sanitized host driver")
    return exe


if __name__ == "__main__":
    print(build_library(verbose=True))
