"""Builds libtdk.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libtdk.so")
SOURCES = [os.path.join(CSRC, "tdk_kernels.hip"), os.path.join(CSRC, "tdk_attend.hip"), os.path.join(CSRC, "tdk_api.cpp"), os.path.join(CSRC, "tdk_plan.cpp"), os.path.join(CSRC, "tdk_prompt.cpp")]
HEADERS = [os.path.join(CSRC, "tdk_internal.h"), os.path.join(CSRC, "tdk_types.h"), os.path.join(CSRC, "tdk_plan.h"), os.path.join(ROOT, "include", "tdk.h"), os.path.join(ROOT, "include", "tdk_bench.h")]


def hipcc_command(out: str = LIB, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "-x", "hip", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
            "-ffp-contract=off",
            # packed fp32 VALU forms are kept out of all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-function",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra, "-o", out, *SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or is_stale():
        cmd = hipcc_command()
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.run(cmd, check=True, cwd=ROOT)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
