"""Builds libl2l.so (HIP kernels + C ABI + host EPS) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libl2l.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
HIPCC = os.path.join(ROCM, "bin", "hipcc")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
             "-Wno-unused-result"]
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-mavx2", "-mfma", "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", "-pthread"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("build failed: " + cmd[0])
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    return r


def build(verbose: bool = False) -> str:
    obj_dir = os.path.join(PKG, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    o_hip = os.path.join(obj_dir, "l2l.o")
    o_eps = os.path.join(obj_dir, "eps.o")
    _run([HIPCC, *HIP_FLAGS, "-c", os.path.join(CSRC, "l2l.hip"), "-o", o_hip])
    _run(["g++", *HOST_FLAGS, "-c", os.path.join(CSRC, "eps.cpp"), "-o", o_eps])
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", o_hip, o_eps, "-o", LIB, "-pthread"])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
