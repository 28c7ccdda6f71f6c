"""Builds the C-ABI library `libregione.so` from csrc/ with hipcc for gfx950, in tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libregione.so")
SOURCES = ["api.hip", "partition.hip", "rows.hip", "gemm.hip", "attention.hip", "block_extras.hip", "fp8.hip", "peaks.hip"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-fno-gpu-rdc",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    # The GEMM's hand-pipelined loads are only correct if the compiler left their registers alone: prove it on the
    # machine code before anything is linked, with the very flags of the build.
    from . import isa_check
    isa_check.check_gemm(hipcc, flags, os.path.join(CSRC, "gemm.hip"))
    cmd = [hipcc, *flags, "-fPIC", "-shared"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("hipcc failed building libregione.so")
    if verbose and proc.stderr:
        sys.stderr.write(proc.stderr)
    return LIB


if __name__ == "__main__":
    sys.path.insert(0, ROOT)
    __package__ = "paper_2510_25590_amd"
    print(build(verbose=True))
