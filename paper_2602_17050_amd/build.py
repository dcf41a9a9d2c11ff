"""Builds libmpzch.so (gfx950) in-tree with hipcc.  `python -m paper_2602_17050_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "mpzch.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "mpzch_kernels.hpp"),
        os.path.join(os.path.dirname(HERE), "include", "mpzch.h")]
LIB = os.path.join(HERE, "libmpzch.so")
CEIL_SRC = os.path.join(HERE, "csrc", "memory_ceilings.hip")
CEIL_BIN = os.path.join(HERE, "memory_ceilings.bin")


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build_library(verbose: bool = False) -> str:
    """Compiles every time it is called (cross-compiles without a GPU)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-result",
           SRC, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_memory_ceilings(verbose: bool = False) -> str:
    """Stand-alone tool that measures the random-access ceilings of the GPU it runs on."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result",
           CEIL_SRC, "-o", CEIL_BIN + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(CEIL_BIN + ".tmp", CEIL_BIN)
    return CEIL_BIN


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
    print(build_memory_ceilings(verbose="-v" in sys.argv))
