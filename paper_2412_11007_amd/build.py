"""Builds libflashsparse_hip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = ["fs_convert.hip", "fs_spmm.hip", "fs_sddmm.hip", "fs_softmax.hip", "fs_attention.hip", "fs_transpose.hip", "fs_api.hip"]
LIB = os.path.join(_HERE, "libflashsparse_hip.so")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source into the in-tree shared library and return its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"),
           # keep the compiler from forming packed-fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + [os.path.join(_HERE, "csrc", s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed with exit code %d" % res.returncode)
    return LIB


EXAMPLE_SRC = os.path.join(ROOT, "tests", "c_abi_example.c")
EXAMPLE_BIN = os.path.join(ROOT, "tests", "c_abi_example")


def build_c_example() -> str:
    """Compile the plain-C program that drives the library through its C ABI (run by a GPU test)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L" + _HERE, "-lflashsparse_hip",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2412_11007_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE_BIN]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
        raise RuntimeError("gcc failed on the C example with exit code %d" % res.returncode)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_example())
