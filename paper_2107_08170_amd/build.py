"""Build the HIP library ``libmv.so`` in-tree for gfx950 (MI355X) with hipcc.

Run ``python -m paper_2107_08170_amd.build``.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libmv.so")
SOURCES = ("csrc/mv_host.hip", "csrc/mv_kernels.hip")
HEADERS = ("csrc/mv_internal.h", "../include/mv.h")


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the HIP library cannot be built")
    return exe


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(os.path.join(PKG_DIR, p)) > t for p in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 into libmv.so (always recompiles)."""
    cmd = [_hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           # packed-FP32 instructions are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
           "-o", LIB_PATH] + [os.path.join(PKG_DIR, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and proc.stderr:
        sys.stderr.write(proc.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
