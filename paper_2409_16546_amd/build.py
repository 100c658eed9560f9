"""Build the HIP library (gfx950) in-tree: ``python -m paper_2409_16546_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libakv.so")
SOURCES = ["akv_api.hip", "akv_append.hip", "akv_decode_split.hip", "akv_decode_head.hip", "akv_fp16.hip", "akw_gemv.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # the decision path is written op by op; FMAs are explicit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 ALU forms on the test machines
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = True, extra: list[str] | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + (extra or []) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
