"""Compile the HIP library (``libaht.so``) for gfx950, in-tree."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("AHT_LIB") or os.path.join(HERE, "libaht.so")
SOURCES = [os.path.join(CSRC, "aht.hip")]
DEPS = SOURCES + [os.path.join(CSRC, "aht_kernels.hpp"), os.path.join(CSRC, "aht_rng.hpp"), os.path.join(CSRC, "aht_mvm.hpp"),
                  os.path.join(os.path.dirname(HERE), "include", "aht.h")]

# Packed fp32 arithmetic is switched off for the device code.  The switch is a cc1 option and the
# driver hands cc1 options to the host pass too, which does not know the feature and says so once
# per invocation; build() drops exactly that line from the log and instead checks the device
# assembly it keeps: no packed fp32 add, multiply or fused multiply-add may appear in it.
PACKED_OFF = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                       # fusion only where the source writes fmaf
    "-fno-fast-math",
    *PACKED_OFF,
    "-Wall", "-Wno-unused-function",
]
# host-side sanitizers (the device code is compiled as always); used by tests/test_sanitizers.py
SANITIZE_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in r.stdout.splitlines() if HOST_NOTE not in l)
    if log.strip():
        print(log, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def build(force: bool = True, verbose: bool = False, extra=(), out: str | None = None) -> str:
    """Compiles the library (to `out`, default in-tree) and checks the device assembly."""
    lib = out or LIB
    if not force and os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(d) for d in DEPS):
        return lib
    with tempfile.TemporaryDirectory(prefix="aht_build_") as tmp:
        staged = os.path.join(tmp, "libaht.so")
        _run([hipcc()] + FLAGS + list(extra) + ["-save-temps=obj", "-o", staged] + SOURCES, verbose)
        asm = [f for f in os.listdir(tmp) if f.endswith(".s") and "amdgcn" in f]
        if not asm:
            raise RuntimeError("the device assembly of the build was not kept: cannot check it")
        packed, lines = 0, 0
        pat = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")
        for f in asm:
            with open(os.path.join(tmp, f), errors="replace") as fh:
                for line in fh:
                    lines += 1
                    packed += bool(pat.search(line))
        if packed:
            raise RuntimeError(f"{packed} packed fp32 instructions in the gfx950 assembly: the switch did not reach the device pass")
        if verbose:
            print(f"device pass: packed fp32 arithmetic off, 0 v_pk_{{add,mul,fma}}_f32 in {lines} lines of gfx950 assembly", flush=True)
        shutil.move(staged, lib)
    return lib


def build_valu_rates() -> str:
    """The instruction issue-rate microbenchmark (measurement support, not part of the library)."""
    out = os.path.join(HERE, "valu_rates")
    _run([hipcc(), "-O3", "--offload-arch=gfx950", *PACKED_OFF, "-o", out, os.path.join(CSRC, "valu_rates.hip")], True)
    return out


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "valu_rates":
        print(build_valu_rates())
    else:
        build(force=True, verbose=True, extra=sys.argv[1:])
        print(LIB)
