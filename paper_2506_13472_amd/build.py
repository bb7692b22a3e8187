"""Builds librosaq.so (host packer + C ABI + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "librosaq.so")
HOST_SOURCES = ["rosaq_pack.cpp", "rosaq_api.cpp"]
HIP_SOURCES = ["rosaq_kernels.hip", "rosaq_pca.hip", "rosaq_static.hip", "rosaq_quant.hip", "rosaq_rotate.hip"]


def hipcc() -> str:
    env = os.environ.get("HIPCC")
    if env:
        return env
    return "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


# The switch that keeps the compiler from forming packed-fp32 instructions is a feature of the gfx950
# target.  hipcc hands -Xclang options to its host pass as well, which does not know the feature and
# says so once per function-multiversioning probe; that line is dropped from the log.  What the
# device pass did is checked instead: its assembly (kept by -save-temps) must hold no packed-fp32
# arithmetic at all.
_HOST_NOISE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
_PK_F32 = re.compile(r"\bv_pk_(?:add|mul|fma)_f32\b")


def _compile_hip(src: str, obj: str, common, verbose: bool) -> None:
    cmd = [hipcc(), "-x", "hip", "--offload-arch=gfx950", "-save-temps=obj",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *common, "-Wno-unused-command-line-argument", "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = [ln for ln in r.stdout.splitlines() if ln.strip() and ln.strip() != _HOST_NOISE]
    if log:
        print("\n".join(log), flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    stem = os.path.splitext(os.path.basename(obj))[0]            # e.g. rosaq_kernels.hip
    stem = os.path.splitext(stem)[0]
    asm = [f for f in os.listdir(os.path.dirname(obj))
           if f.startswith(stem + "-hip-amdgcn") and f.endswith(".s")]
    if not asm:
        raise RuntimeError(f"no device assembly kept for {src}")
    n = 0
    for f in asm:
        with open(os.path.join(os.path.dirname(obj), f), "r", errors="replace") as fh:
            n += len(_PK_F32.findall(fh.read()))
    print(f"{os.path.basename(src)}: device pass for gfx950 holds {n} packed-fp32 instructions", flush=True)
    if n:
        raise RuntimeError(f"{src}: packed-fp32 arithmetic in the device code")


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC,
              "-I", os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "include")]
    jobs = []
    objs = []
    for s in HOST_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        jobs.append((_run, ([hipcc(), "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-pthread", *common,
                             "-c", os.path.join(CSRC, s), "-o", o], verbose)))
        objs.append(o)
    for s in HIP_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        jobs.append((_compile_hip, (os.path.join(CSRC, s), o, common, verbose)))
        objs.append(o)
    # the translation units are independent: compile them side by side
    with ThreadPoolExecutor(max_workers=min(len(jobs), max(1, (os.cpu_count() or 2) // 2))) as ex:
        for f in [ex.submit(fn, *a) for fn, a in jobs]:
            f.result()
    _run([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-pthread", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
