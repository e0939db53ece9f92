"""Compile libelmrnn.so (HIP, gfx950) in-tree.  Usage: python -m paper_1911_13252_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libelmrnn.so")
SOURCES = ("api.hip", "hidden.hip", "hidden_fused.hip", "hidden_split.hip", "hidden_tiny.hip", "hidden_diag.hip", "hidden_fc.hip", "specrad.hip", "tsqr.hip", "solve.hip", "solve_static.hip", "probe.hip")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(src: str, extra=()) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.run(cmd, check=True)
    return obj


def build_library(verbose: bool = False, extra=(), out: str = LIB_PATH) -> str:
    """Compile every source for gfx950 and link the shared library; returns its path."""
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, extra), SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs],
                   check=True)
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build_library(verbose=True, extra=tuple(sys.argv[1:]))
