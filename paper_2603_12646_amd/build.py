"""Builds libfa_mi355x.so (HIP kernels + C boundary) in-tree for gfx950.

Usage: python -m paper_2603_12646_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_NAME = "libfa_mi355x.so"
LIB_PATH = os.path.join(HERE, LIB_NAME)
SOURCES = [os.path.join(HERE, "csrc", "fa_kernels.hip"), os.path.join(HERE, "csrc", "fa_api.cpp")]
# standalone measurement program (matrix-core and copy ceilings); bench.py runs it as a child
CEILINGS_SRC = os.path.join(HERE, "csrc", "ceilings.hip")
CEILINGS_PATH = os.path.join(HERE, "fa_ceilings")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(HERE, "csrc"), "-x", "hip", *SOURCES, "-o", LIB_PATH]
    if verbose:
        print("+", " ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{err}")
    return LIB_PATH


def build_ceilings(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc, *flags, "-x", "hip", CEILINGS_SRC, "-o", CEILINGS_PATH]
    if verbose:
        print("+", " ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{proc.stderr}")
    return CEILINGS_PATH


if __name__ == "__main__":
    print(build_library())
    print(build_ceilings())
