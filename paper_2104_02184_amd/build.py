"""Compile the HIP library (``libaht.so``) for gfx950, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaht.so")
SOURCES = [os.path.join(CSRC, "aht.hip")]
DEPS = SOURCES + [os.path.join(CSRC, "aht_kernels.hpp"), os.path.join(CSRC, "aht_rng.hpp"), os.path.join(CSRC, "aht_mvm.hpp"),
                  os.path.join(os.path.dirname(HERE), "include", "aht.h")]

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                       # fusion only where the source writes fmaf
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def build(force: bool = True, verbose: bool = False, extra=()) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    cmd = [hipcc()] + FLAGS + list(extra) + ["-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def build_valu_rates() -> str:
    """The instruction issue-rate microbenchmark (measurement support, not part of the library)."""
    out = os.path.join(HERE, "valu_rates")
    cmd = [hipcc(), "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", out, os.path.join(CSRC, "valu_rates.hip")]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "valu_rates":
        print(build_valu_rates())
    else:
        build(force=True, verbose=True, extra=sys.argv[1:])
        print(LIB)
