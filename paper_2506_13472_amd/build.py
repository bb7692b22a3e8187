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


PROBES = ("EMPTY", "NO_X", "NO_W", "NO_COMPUTE", "NO_EPI", "TIMELINE")


def build_probe(names, verbose: bool = True) -> str:
    """A measurement variant of the library next to the real one: `gemm_kernel` compiled with
    -DROSAQ_PROBE_<NAME> for every name given (e.g. NO_COMPUTE: loads only; TIMELINE: per-wave clock
    stamps read back through rosaq_debug_timeline).  Results of such a library are not valid outputs.
    Load it by pointing the environment variable ROSAQ_LIB at the returned path.  Needs a prior build()."""
    for n in names:
        if n not in PROBES:
            raise ValueError(f"unknown probe {n!r}; choose from {PROBES}")
    out = os.path.join(PKG, "librosaq_probe_" + "_".join(names) + ".so")
    obj = os.path.join(OBJ, "rosaq_kernels.probe_" + "_".join(names) + ".o")
    _run([hipcc(), "-x", "hip", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          *[f"-DROSAQ_PROBE_{n}" for n in names], "-c", os.path.join(CSRC, "rosaq_kernels.hip"), "-o", obj],
         verbose)
    others = [os.path.join(OBJ, s + ".o") for s in HOST_SOURCES + ["rosaq_pca.hip"]]
    _run([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-pthread", *others, obj, "-o", out], verbose)
    return out


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
    import sys
    build()
    print("built", LIB)
    if len(sys.argv) > 2 and sys.argv[1] == "--probe":
        print("built", build_probe(sys.argv[2].split("+")))
