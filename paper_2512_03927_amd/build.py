"""Builds libodmoe.so (HIP, gfx950) and libodmoe_hostsim.so (host-only) in-tree.

    python -m paper_2512_03927_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libodmoe.so")
HOSTSIM = os.path.join(PKG, "libodmoe_hostsim.so")
C_DEMO = os.path.join(PKG, "c_abi_demo")   # plain C program on top of the C ABI (run by a GPU test)

HIP_SOURCES = ["odmoe_api.hip", "decode_kernels.hip", "quant_kernels.hip", "quant4_kernels.hip", "f16_kernels.hip", "prefill_kernels.hip"]
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms have produced wrong results on these machines: keep them off
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd):
    print("+", " ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in HIP_SOURCES]
    _run([hipcc, *HIP_FLAGS, *srcs, "-o", LIB])
    _run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall",
          os.path.join(CSRC, "hosttest_api.cpp"), "-o", HOSTSIM])
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    _run(["gcc", "-O2", "-std=c11", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
          "-I" + os.path.join(os.path.dirname(PKG), "include"), os.path.join(CSRC, "c_abi_demo.c"),
          "-L" + PKG, "-lodmoe", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
          "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", C_DEMO])
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
