"""Builds the HIP library in-tree: paper_1805_10692_amd/libcer_hip.so (gfx950 only).

    python -m paper_1805_10692_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcer_hip.so")
SOURCES = ["cer_host.cpp", "cer_capi.cpp", "cer_gemv.hip", "cer_gemm.hip", "cer_xtile.hip", "cer_strip.hip", "cer_matmul.hip", "dense_kernels.hip", "csr.hip", "cost_model.cpp", "frontend.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         # fp32 division rounds correctly (the quantizer's codes must equal a binary32 reference bit for bit)
         "-fhip-fp32-correctly-rounded-divide-sqrt",
         # packed-fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the first 16 dwords of a kernel's arguments arrive in scalar registers with the wave (kernels whose leading
         # arguments are plain pointers and integers start without waiting for a load of their arguments)
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return obj


def build_library(verbose: bool = True) -> str:
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES))  # every source is compiled on every call
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", tmp, "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
