"""Builds liblmhead.so (HIP, gfx950 only) next to this file.

Usage: ``python -m paper_2603_04411_amd.build`` or ``build_library()``.
hipcc cross-compiles without a GPU present.

``python -m paper_2603_04411_amd.build --trace`` builds liblmhead_trace.so instead: the same sources with
-DLMHEAD_TRACE, i.e. with per-workgroup time stamps in the forward kernel (read by ``tile_trace.py``; a
diagnostic build, never loaded by the binding).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblmhead.so")
TRACE_LIB = os.path.join(HERE, "liblmhead_trace.so")
SOURCES = ["lmhead_api.hip", "lmhead_aux.hip", "lmhead_loss.hip", "lmhead_gemm.hip", "lmhead_probe.hip",
           "dynakv_api.hip", "dynakv_aux.hip", "dynakv_gemm.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed fp32 VALU forms are kept off for every device translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(verbose: bool = False, trace: bool = False) -> str:
    objdir = os.path.join(HERE, "_build_trace" if trace else "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()
    flags = FLAGS + (["-DLMHEAD_TRACE"] if trace else [])
    lib = TRACE_LIB if trace else LIB

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return lib


if __name__ == "__main__":
    print(build_library(verbose=True, trace="--trace" in sys.argv[1:]))
