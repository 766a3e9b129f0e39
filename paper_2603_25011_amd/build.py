"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "liblsr_head.so")
SRC = os.path.join(PKG, "csrc", "lsr_head.hip")
# benchmark comparator (the reduce step of the paper's hybrid forward); not part of the product library
ALG2_LIB = os.path.join(PKG, "libalg2_reduce.so")
ALG2_SRC = os.path.join(PKG, "csrc", "alg2_reduce.hip")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    # packed-fp32 instruction forms are switched off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def _compile(src: str, lib: str, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
           "-o", lib, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError(f"hipcc failed building {os.path.basename(lib)}")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)


def build(verbose: bool = False) -> str:
    _compile(SRC, LIB, verbose)
    _compile(ALG2_SRC, ALG2_LIB, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
