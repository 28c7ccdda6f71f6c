"""Builds the C-ABI library `libregione.so` from csrc/ with hipcc for gfx950, in tree.

Every source is compiled to its own object (in parallel, objects under csrc/_build/) and the objects are linked
into the shared library; `build()` always compiles everything again."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libregione.so")
SOURCES = ["api.hip", "partition.hip", "rows.hip", "gemm.hip", "attention.hip", "block_extras.hip", "fp8.hip", "peaks.hip",
           "fp32.hip", "host_logic.cpp"]


def flags() -> list[str]:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-Wno-inline-asm", "-fno-gpu-rdc",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError(f"hipcc failed: {' '.join(cmd[-3:])}")
    if verbose and proc.stderr:
        # the host pass does not know the packed-fp32 target feature and says so once per file: harmless
        sys.stderr.write("".join(l for l in proc.stderr.splitlines(True) if "packed-fp32-ops" not in l))


def build(verbose: bool = False, only=None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    fl = flags()
    os.makedirs(OBJ, exist_ok=True)
    sources = [s for s in SOURCES if only is None or s in only]
    if only is not None:   # a partial build is only sound while no header is newer than the objects that are kept
        headers = [os.path.join(CSRC, "common.h")] + [os.path.join(ROOT, "include", h) for h in os.listdir(os.path.join(ROOT, "include"))]
        newest = max(os.path.getmtime(h) for h in headers)
        kept = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES if s not in sources]
        if any(not os.path.exists(o) or os.path.getmtime(o) < newest for o in kept):
            sources = list(SOURCES)

    def compile_one(src):
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        _run([hipcc, *fl, "-fPIC", "-c", os.path.join(CSRC, src), "-o", obj], verbose)
        return obj

    def check_isa(_):
        # The GEMM's hand-pipelined loads are only correct if the compiler left their registers alone: prove it on the
        # machine code before anything is linked, with the very flags of the build.
        from . import isa_check
        isa_check.check_gemm(hipcc, fl, os.path.join(CSRC, "gemm.hip"))

    jobs = int(os.environ.get("MAX_JOBS", "8"))
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, 16))) as pool:
        futs = [pool.submit(compile_one, s) for s in sources]
        if only is None or "gemm.hip" in only:
            futs.append(pool.submit(check_isa, None))
        for f in futs:
            f.result()
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    _run([hipcc, *fl, "-fPIC", "-shared", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    sys.path.insert(0, ROOT)
    __package__ = "paper_2510_25590_amd"
    only = sys.argv[1:] or None
    print(build(verbose=True, only=only))
