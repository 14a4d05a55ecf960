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

SOURCES = ["tova_kernels.hip", "tova_prefill.hip", "tova_repos.hip", "tova_policy.hip", "tova_static_scratch.hip",
           "tova_api.cpp"]

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


def build(verbose: bool = True, extra_flags=(), jobs: int = 8) -> str:
    """Compiles every source (always: nothing is reused from an earlier build), the translation
    units side by side, then links them into libtova.so."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="libtova_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc(), *flags, *extra_flags, *inc, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
