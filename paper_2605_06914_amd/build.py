"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libtaper_attn.so")
SOURCES = ["taper_kernels.hip", "taper_static.hip", "taper_api.cpp", "taper_plan.cpp", "taper_admission.cpp"]
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
    # never let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


TRACE_LIB = os.path.join(PKG, "libtaper_attn_trace.so")  # development aid: per-workgroup clocks (wg_trace.py)


def build_library(verbose: bool = False, extra_flags=(), trace: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if trace:
        return _build(hipcc, TRACE_LIB, ["-DTAPER_WG_TRACE", *extra_flags], verbose)
    return _build(hipcc, LIB, list(extra_flags), verbose)


def _build(hipcc, lib, extra_flags, verbose) -> str:
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIP_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", tmp, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    args = sys.argv[1:]
    print(build_library(verbose=True, extra_flags=[a for a in args if a != "--trace"], trace="--trace" in args))
