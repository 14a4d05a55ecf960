"""Builds libtova.so (the C-ABI library) in-tree with hipcc for gfx950.

    python -m paper_2401_06104_amd.build

The library is not built on import: tests, the smoke check and the benchmark load what is
there and fail loudly when it is missing.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libtova.so")

SOURCES = ["tova_kernels.hip", "tova_prefill.hip", "tova_repos.hip", "tova_policy.hip", "tova_api.cpp"]

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; a ROCm toolchain is required to build libtova.so")
    return exe


def build(verbose: bool = True, extra_flags=()) -> str:
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
