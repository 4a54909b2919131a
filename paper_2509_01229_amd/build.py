"""Build the C-ABI library paper_2509_01229_amd/libliquidgemm.so with hipcc for gfx950.

`python -m paper_2509_01229_amd.build` compiles csrc/*.hip and csrc/*.cpp in-tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libliquidgemm.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ["liquidgemm.hip", "actquant.hip", "calib.hip", "lqq_pack.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep hipcc from forming packed-FP32 instructions out of ordinary float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-lpthread",
]


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", out, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libliquidgemm.so")
    if verbose and res.stderr:
        sys.stderr.write(res.stderr)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
