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
SOURCES = ["host_ops.cpp", "quantize.hip", "attention.hip", "decode_mfma.hip", "decode_mfma_p8.hip", "decode_rope.hip", "measure.hip"]

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


def build_library(verbose: bool = True, extra_flags=(), jobs: int = 6) -> str:
    """Compiles every source to an object file (in parallel, in a scratch directory beside the library)
    and links them into libkvbfp.so."""
    import concurrent.futures
    import tempfile
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="_build_", dir=PKG) as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc_path(), *compile_flags, *extra_flags, *inc, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    build_library()
    print("built", LIB)
    sys.exit(0)
