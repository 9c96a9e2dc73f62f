"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libconv2d_int8.so")
SOURCES = ["api.cpp", "selector.cpp", "igemm_mfma.hip", "band_mfma.hip", "layout_kernels.hip", "window_mfma.hip",
           "pointwise_mfma.hip"]
HEADERS = [os.path.join(CSRC, "kernels.h"), os.path.join(CSRC, "rewrite_bodies.h"), os.path.join(CSRC, "act_requant.h"), os.path.join(CSRC, "desc_check.h"),
           os.path.join(os.path.dirname(PKG), "include", "conv2d_int8.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    "-Wno-unused-command-line-argument",
    # keep the compiler from forming packed-fp32 ALU ops (harmless host-side warning)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(verbose: bool = False) -> str:
    from concurrent.futures import ThreadPoolExecutor

    def compile_one(s):
        src = os.path.join(CSRC, s)
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        cmd = ["hipcc", *HIPCC_FLAGS, "-x", "hip", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    # the translation units are independent: compile them side by side (the GEMM kernel's file dominates)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
    print(LIB)
    sys.exit(0)
