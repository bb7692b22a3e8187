"""Builds librosaq.so (host packer + C ABI + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "librosaq.so")
HOST_SOURCES = ["rosaq_pack.cpp", "rosaq_api.cpp"]
HIP_SOURCES = ["rosaq_kernels.hip", "rosaq_pca.hip"]


def hipcc() -> str:
    env = os.environ.get("HIPCC")
    if env:
        return env
    return "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC,
              "-I", os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "include")]
    objs = []
    for s in HOST_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        _run([hipcc(), "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-pthread", *common,
              "-c", os.path.join(CSRC, s), "-o", o], verbose)
        objs.append(o)
    for s in HIP_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        _run([hipcc(), "-x", "hip", "--offload-arch=gfx950",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              *common, "-c", os.path.join(CSRC, s), "-o", o], verbose)
        objs.append(o)
    _run([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-pthread", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
