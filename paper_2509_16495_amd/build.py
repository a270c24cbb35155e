"""Builds libshiftattn.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libshiftattn.so")
SOURCES = ["api.hip", "layout_kernels.hip", "attn_generic.hip", "decode_mfma.hip", "prefill_mfma.hip", "prefill_mfma64.hip", "ceilings.hip", "proj_gemm.hip", "proj_stream.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False, extra: list[str] | None = None) -> str:
    cmd = ["hipcc", *FLAGS, *(extra or []), "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True, extra=sys.argv[1:])
