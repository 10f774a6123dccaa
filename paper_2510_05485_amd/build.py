"""Build the gfx950 shared library (libtensorbleu.so) in-tree with hipcc.

`python -m paper_2510_05485_amd.build` compiles every HIP translation unit under csrc/ for
gfx950 and links them into one C-ABI library next to this file.  hipcc cross-compiles without a
GPU, so this runs anywhere the ROCm toolchain is installed.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libtensorbleu.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = True) -> str:
    tmp = LIB + f".tmp{os.getpid()}"
    extra = os.environ.get("TB_HIPCC_EXTRA", "").split()   # extra hipcc flags for experiments
    cmd = [HIPCC, *FLAGS, *extra, "-I", INCLUDE, "-I", CSRC, "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


EXAMPLE_SRC = os.path.join(PKG, "example", "c_caller.c")
EXAMPLE_BIN = os.path.join(PKG, "c_caller")


def build_example(verbose: bool = True) -> str:
    """The plain-C caller of the ABI (gcc, HIP runtime only), linked against the library."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c99", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__",
           "-I", INCLUDE, "-I", os.path.join(rocm, "include"), EXAMPLE_SRC, "-L", PKG,
           "-ltensorbleu", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return EXAMPLE_BIN


if __name__ == "__main__":
    build()
    build_example()
    print("built", LIB)
    sys.exit(0)
