"""Builds libbspmm.so (HIP kernels + scheduler + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbspmm.so")
SOURCES = ["kernels.hip", "schedule.cpp", "api.cpp"]
HEADERS = ["plan.hpp", "schedule.hpp", os.path.join("..", "..", "include", "bspmm.h")]


def lib_path() -> str:
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # kernels whose arguments are plain pointers and integers get them in SGPRs when a
           # wavefront starts (the command processor fills up to 16 of them): their first
           # dependent fetch, the work item, goes out at once instead of after a kernel-argument
           # load
           "-mllvm", "-amdgpu-kernarg-preload-count=16",
           "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
           "-x", "hip", os.path.join(CSRC, "kernels.hip"),
           "-x", "hip", os.path.join(CSRC, "schedule.cpp"),
           "-x", "hip", os.path.join(CSRC, "api.cpp"),
           "-o", LIB]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout)
    if verbose and r.stdout.strip():
        print(r.stdout, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
