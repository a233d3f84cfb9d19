"""Builds libfastgen.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfastgen.so")
SOURCES = ["fastgen_api.hip", "profile_mfma.hip", "profile_f32.hip", "select.hip", "decode.hip"]
# measurement aid of bench.py (micro-benchmarks of the matrix and vector pipes), its own library
UBENCH_LIB = os.path.join(HERE, "libfgubench.so")
UBENCH_SOURCES = ["ubench.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 VALU forms stay off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no kernel produces or tests for a NaN; without this every fmaxf on a matrix-core result is
    # preceded by an instruction that quiets a signalling NaN (three per owner fragment and tile
    # in the first profiling sweep)
    "-fno-honor-nans",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the FastGen library needs ROCm to build")
    return exe


def _compile(sources, lib, verbose):
    cmd = [hipcc(), *FLAGS, *[os.path.join(CSRC, s) for s in sources], "-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = True) -> str:
    _compile(SOURCES, LIB, verbose)
    _compile(UBENCH_SOURCES, UBENCH_LIB, verbose)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
