"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeager.so")
SOURCES = ["eager_round_kernels.hip", "eager_chunk_kernels.hip", "eager_aux_kernels.hip",
           "eager_api.cpp"]

# -ffp-contract=off: the fixed-order mode defines every rounding; fused multiply-adds are
# written out where they are meant.  Packed fp32 instructions are switched off.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, "-x", "hip",
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def ensure_built() -> str:
    """For the test suite, the smoke run and the benchmark: compile only if no library has
    been built yet (the binding itself never builds: without a library it raises)."""
    return LIB if os.path.exists(LIB) else build(verbose=True)


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
