"""Builds librekv.so (the C-ABI library of HIP kernels) for gfx950, in-tree, and the C test program.

    python -m paper_2503_00540_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "librekv.so")
SOURCES = ["api.hip", "attention_bf16.hip", "attention_f32.hip", "retrieval.hip", "gather.hip", "probe.hip"]

# Packed-fp32 VALU instructions are switched off for all device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build_library(verbose: bool = True, extra: list[str] | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *(extra or []), *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


C_PROGRAM_SRC = os.path.join(ROOT, "tests", "abi_chain.c")
C_PROGRAM = os.path.join(ROOT, "tests", "abi_chain")


def build_c_program(verbose: bool = True) -> str:
    """The plain C99 program that drives the whole path through the C ABI (tests/abi_chain.c):
    host compiler only, linked against librekv.so and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), C_PROGRAM_SRC,
           "-L", PKG, "-l:librekv.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2503_00540_amd", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}", "-o", C_PROGRAM]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_PROGRAM


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
    build_c_program()
