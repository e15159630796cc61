"""Builds libtmac_hip.so (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libtmac_hip.so")
SOURCES = ["tmac_kernels.hip", "tmac_perm.hip", "tmac_rows.hip", "tmac_noalloc.hip", "tmac_pack.cpp"]
# measurement helpers (plain read, LDS probe, empty kernel): a library of their own, not the product's ABI
BENCH_LIB_PATH = os.path.join(PKG_DIR, "libtmac_bench.so")
BENCH_SOURCES = ["tmac_bench.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the first eight dwords of a kernel's arguments arrive in scalar registers when a wave starts
    # (the decode kernel's leading integer arguments: which matrix a workgroup serves is then known
    # without a trip to memory; one launch for three matrices: 13.95 -> 13.70 us)
    "-mllvm", "-amdgpu-kernarg-preload-count=8",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _compile(out: str, sources, verbose: bool, extra_flags=()) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-o", out]
    for s in sources:
        path = os.path.join(CSRC, s)
        cmd += ["-x", "hip", path] if s.endswith(".cpp") else [path]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True, extra_flags=()) -> str:
    _compile(LIB_PATH, SOURCES, verbose, extra_flags)
    _compile(BENCH_LIB_PATH, BENCH_SOURCES, verbose, extra_flags)
    return LIB_PATH


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
