"""Builds the HIP library for gfx950 in-tree: paper_2604_06483_amd/libll.so.

    python -m paper_2604_06483_amd.build

hipcc cross-compiles without a GPU.  The packed-fp32 instructions are switched off for all
device code.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["ll_api.hip", "ll_project.hip", "ll_steer.hip", "ll_capture.hip"]
LIB = os.path.join(HERE, "libll.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def build(verbose: bool = True, extra_flags=()) -> str:
    srcs = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd = ["hipcc", *FLAGS, *extra_flags, *srcs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless noise.
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}\n{res.stderr}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
    print("built", LIB)
