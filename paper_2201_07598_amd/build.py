"""Build libokt.so (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2201_07598_amd.build

hipcc cross-compiles without a GPU.  The library lands next to this file so
that it travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libokt.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # the accumulate must round the product and the sum separately
    "-ffp-contract=off",
    # keep subnormals (the default), and no packed fp32 arithmetic
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


CABI_SMOKE_SRC = os.path.join(ROOT, "tests", "cabi", "cabi_smoke.cpp")
CABI_SMOKE_BIN = os.path.join(ROOT, "tests", "cabi", "cabi_smoke.bin")


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    sources = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(HERE, "csrc"), *sources, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    build_cabi_smoke(verbose)
    return LIB


def build_cabi_smoke(verbose: bool = True, out: str = CABI_SMOKE_BIN) -> str:
    """The host program of tests/cabi: a plain C++ caller of the C ABI (hipMalloc,
    default stream, no Python), linked against the library next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"),
           CABI_SMOKE_SRC, "-L", HERE, "-lokt", "-Wl,-rpath," + HERE,
           "-Wl,-rpath,$ORIGIN/../../paper_2201_07598_amd", "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)
