"""Builds the gfx950 C-ABI library in-tree with hipcc (no torch extension machinery)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libernie_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # only the C entry points (marked ERNIE_API in include/*.h) leave the library
    "-fvisibility=hidden", "-fvisibility-inlines-hidden",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = True) -> str:
    """Compile csrc/ernie_api.hip, csrc/prune_api.hip and csrc/job_api.hip (which include every kernel header) into libernie_hip.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, "ernie_api.hip"), os.path.join(CSRC, "prune_api.hip"), os.path.join(CSRC, "job_api.hip"),
                                "-Wl,--version-script=" + os.path.join(CSRC, "exports.map"), "-lpthread", "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass prints a harmless note that it does not know the packed-fp32 feature
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    return LIB_PATH


if __name__ == "__main__":
    build_library()
