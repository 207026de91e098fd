"""Builds libslkv.so (HIP kernels for gfx950 + the C ABI) in-tree with hipcc.

Usage: python -m paper_2508_15806_amd.build
"""

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libslkv.so")

ROCM_INCLUDE = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "include")

HIP_SOURCES = ["compress.hip", "stage1.hip"]
HOST_SOURCES = ["slkv_host.cpp", "timing.cpp"]

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# packed fp32 VALU ops are kept off for device code
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def run(cmd):
    print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    for src in HIP_SOURCES:
        obj = os.path.join(objdir, src + ".o")
        run([hipcc] + COMMON + DEVICE + ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in HOST_SOURCES:
        obj = os.path.join(objdir, src + ".o")
        # plain C++ (no device pass); host arithmetic (budget allocation) must not be contracted into FMAs
        run([hipcc] + COMMON + ["-ffp-contract=off", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", ROCM_INCLUDE, "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
