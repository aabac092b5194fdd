"""Builds libflce.so (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2511_17599_amd.build

hipcc cross-compiles without a GPU.  The packed-fp32 target feature is switched
off for all device code of this library.
"""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(PKG, "csrc", "flce.hip")
LIB = os.path.join(PKG, "libflce.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc_path():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose=False):
    """Compiles csrc/flce.hip into libflce.so next to this file; returns its path."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, SRC, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
