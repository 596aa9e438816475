"""Builds the C-ABI library (HIP kernels for gfx950 + host pattern compiler) in-tree.

    python -m paper_2506_03065_amd.build

produces paper_2506_03065_amd/libsparse_vdit.so with hipcc.  hipcc cross-compiles
gfx950 code objects without a GPU present.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libsparse_vdit.so")
SOURCES = ["attn_kernels.hip", "fp8_kernels.hip", "search_kernels.hip", "rearrange_kernels.hip", "static_scratch.hip", "probe_kernels.hip", "api.cpp", "pattern_compiler.cpp"]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; the library cannot be built")


def build_library(verbose: bool = True) -> str:
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-x", "hip",
           # NaNs need no special care in fmax chains (infinities stay honoured: masks use -inf)
           "-fno-honor-nans",
           # packed fp32 VALU forms are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library())
