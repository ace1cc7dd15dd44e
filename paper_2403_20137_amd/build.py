"""Builds libkvbfp.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2403_20137_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libkvbfp.so")
SOURCES = ["host_ops.cpp", "quantize.hip", "attention.hip", "decode_mfma.hip", "decode_mfma_p8.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def hipcc_path() -> str:
    cand = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(cand):
        raise RuntimeError("hipcc not found; libkvbfp needs the ROCm toolchain")
    return cand


def build_library(verbose: bool = True, extra_flags=()) -> str:
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".hip") else ["-x", "hip", path])
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_library()
    print("built", LIB)
    sys.exit(0)
