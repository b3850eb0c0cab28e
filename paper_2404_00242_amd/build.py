"""Builds libdeft.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""

from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdeft.so")
SOURCES = ["deft_plan.cpp", "deft_decode.hip"]


def hipcc_command(out: str = LIB, extra=()):
    return [
        "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        # packed-FP32 VALU forms are kept out of the generated code on purpose
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        *extra, *os.environ.get("DEFT_EXTRA_FLAGS", "").split(),
        *[os.path.join(CSRC, s) for s in SOURCES],
        "-o", out,
    ]


def build_library(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
