"""Builds libflashsparse_hip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = ["fs_convert.hip", "fs_spmm.hip", "fs_sddmm.hip", "fs_softmax.hip", "fs_attention.hip", "fs_transpose.hip", "fs_api.hip"]
LIB = os.path.join(_HERE, "libflashsparse_hip.so")
OBJ_DIR = os.path.join(_HERE, "_build")  # object files; ignored by git
# k_sddmm uses its matrix-core results at once: let them land in ordinary vector registers instead of
# accumulation registers that eight copy instructions per block would have to read back (the other kernels
# get this form from the compiler unasked)
FILE_FLAGS = {"fs_sddmm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("%s failed with exit code %d" % (os.path.basename(cmd[0]), res.returncode))


def build_library(verbose: bool = False, defines=(), lib: str = LIB) -> str:
    """Compile every HIP source (one hipcc process per file, side by side) and link the in-tree shared
    library; returns its path.  ``defines`` adds -D flags (e.g. a debug build under another ``lib`` name)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = OBJ_DIR if lib == LIB else lib + ".objs"
    os.makedirs(obj_dir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-I" + os.path.join(ROOT, "include"),
             # keep the compiler from forming packed-fp32 instructions
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + ["-D" + d for d in defines]
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc] + flags + FILE_FLAGS.get(s, []) + ["-c", os.path.join(_HERE, "csrc", s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs, verbose)
    return lib


EXAMPLE_SRC = os.path.join(ROOT, "tests", "c_abi_example.c")
EXAMPLE_BIN = os.path.join(ROOT, "tests", "c_abi_example")


def build_c_example() -> str:
    """Compile the plain-C program that drives the library through its C ABI (run by a GPU test)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L" + _HERE, "-lflashsparse_hip",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2412_11007_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE_BIN]
    _run(cmd, False)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_example())
