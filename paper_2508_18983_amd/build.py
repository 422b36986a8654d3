"""Compile libsmoe.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsmoe.so")
HOSTLOGIC_LIB = os.path.join(PKG, "libsmoe_hostlogic.so")
SOURCES = ["smoe_host.hip", "route_kernel.hip", "ffn_kernels.hip"]
BUILD_DIR = os.path.join(PKG, "_build")


def build_library(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    gxx = shutil.which("g++") or "g++"
    # host-core expert FFN (CPU-assisted scheduling): host-only C++, built by g++ so that
    # its loops get AVX-512 / AVX2 / baseline versions selected at load time
    os.makedirs(BUILD_DIR, exist_ok=True)
    cpu_obj = os.path.join(BUILD_DIR, "cpu_expert.o")
    cmd = [gxx, "-O3", "-std=c++17", "-fPIC", "-pthread", "-Wall", "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, "-c", os.path.join(CSRC, "cpu_expert.cpp"), "-o", cpu_obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=ROOT)
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES] + ["-Wl," + cpu_obj, "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=ROOT)
    # CPU-only shim around the cache bookkeeping, for the tests that run without a GPU
    cmd = [gxx, "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", "-Wall", "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, "-o", HOSTLOGIC_LIB, os.path.join(CSRC, "hostlogic_shim.cpp"), cpu_obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=ROOT)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
