"""Builds libl2l.so (HIP kernels + C ABI + host EPS) for gfx950, in-tree."""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libl2l.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
HIPCC = os.path.join(ROCM, "bin", "hipcc")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
             "-munsafe-fp-atomics",      # fp32 atomics on device memory go to the hardware atomic units
             "-Wno-unused-result"] + os.environ.get("L2L_EXTRA_HIPFLAGS", "").split()   # (experiments: extra -D switches)
with open(os.path.join(CSRC, "gemm_variants.h")) as _f:
    NUM_GEMM_VARIANTS = int(re.search(r"kNumGemmVariants\s*=\s*(\d+)", _f.read()).group(1))
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-mavx2", "-mfma", "-mf16c", "-fno-math-errno", "-fopenmp-simd",   # (sqrt without errno, simd reductions: the optimizer loops vectorise)
              "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", "-pthread"]


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
    jobs = [[HIPCC, *HIP_FLAGS, "-c", os.path.join(CSRC, "l2l.hip"), "-o", o_hip],
            ["g++", *HOST_FLAGS, "-c", os.path.join(CSRC, "eps.cpp"), "-o", o_eps]]
    objs = [o_hip, o_eps]
    for v in range(NUM_GEMM_VARIANTS):        # one translation unit per MFMA tile variant and 16-bit format
        for tag, extra in (("v", []), ("h", ["-DL2L_ELEM_FP16=1"])):
            o = os.path.join(obj_dir, f"gemm_{tag}{v}.o")
            jobs.append([HIPCC, *HIP_FLAGS, f"-DL2L_VARIANT={v}", *extra, "-c", os.path.join(CSRC, "gemm_variant.hip"), "-o", o])
            objs.append(o)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        list(ex.map(_run, jobs))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB, "-pthread"])
    if verbose:
        print("built", LIB)
    return LIB


def build_host_sanitized(kind: str, driver: str, out: str) -> str:
    """Host-only build of the EPS (csrc/eps.cpp) together with a driver program, under a sanitizer:
    kind = "address,undefined" or "thread".  No GPU code and no GPU runtime is linked: the driver defines the few HIP
    runtime functions the EPS calls.  Returns the path of the executable."""
    if kind not in ("address,undefined", "thread"):
        raise ValueError("sanitizer: 'address,undefined' or 'thread'")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    _run(["g++", "-O1", "-g", "-std=c++17", "-mavx2", "-mfma", "-mf16c", "-fopenmp-simd", f"-fsanitize={kind}", "-fno-omit-frame-pointer",
          "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", os.path.join(CSRC, "eps.cpp"), driver, "-o", out, "-pthread"])
    return out


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1].startswith("--sanitize="):
        # python -m paper_2002_05645_amd.build --sanitize=thread  (or address,undefined): builds and runs the EPS driver
        kind = sys.argv[1].split("=", 1)[1]
        root = os.path.dirname(PKG)
        exe = build_host_sanitized(kind, os.path.join(root, "tests", "host", "eps_threads_driver.cpp"),
                                   os.path.join(PKG, "_build", "eps_threads_" + kind.replace(",", "_")))
        sys.exit(subprocess.run([exe]).returncode)
    build(verbose=True)
