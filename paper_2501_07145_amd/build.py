"""Builds librfsf_ts.so in-tree with hipcc for gfx950 (no GPU needed: cross-compiles)."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "librfsf_ts.so")
SOURCES = ["rfsf_ts_api.hip", "rff_increments.hip", "sketch_fft_scan.hip", "gram.hip", "normalize.hip", "dp1d.hip", "trp.hip", "join_pieces.hip", "probe.hip"] + \
    [f"sketch_fft_scan_d{n}.hip" for n in [6, 7, 8, 9, 10, 12, 13, 100, 200, 500, 1000, 2048]]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-command-line-argument",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


EXTRA = os.environ.get("RFSF_EXTRA_HIPCC_FLAGS", "").split()   # extra compiler flags for experiments


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *FLAGS, *EXTRA, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library. Always recompiles."""
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(os.cpu_count() or 4, 16, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
