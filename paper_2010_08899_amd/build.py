"""Builds the HIP libraries (gfx950 only) in-tree with hipcc:
libdct.so, the product (every csrc/*.hip), and libdct_bench.so, the plain streaming
kernels that only bench.py loads (csrc/bench/*.hip)."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdct.so")
BENCH_LIB = os.path.join(PKG, "libdct_bench.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def bench_sources():
    return sorted(glob.glob(os.path.join(CSRC, "bench", "*.hip")))


def _stale(lib: str, srcs) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    deps = list(srcs) + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def needs_build() -> bool:
    return _stale(LIB, sources()) or _stale(BENCH_LIB, bench_sources())


def _compile(lib: str, srcs, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", lib, *srcs]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every kernel for gfx950: the product library and the benchmark's probe library."""
    if force or _stale(LIB, sources()):
        _compile(LIB, sources(), verbose)
    if force or _stale(BENCH_LIB, bench_sources()):
        _compile(BENCH_LIB, bench_sources(), verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
