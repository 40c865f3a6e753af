"""Builds libcomp_ams.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcomp_ams.so")
SOURCES = [os.path.join(CSRC, "comp_ams.hip")]
HEADERS = [os.path.join(CSRC, f) for f in ("device_utils.h", "blocksign_kernels.h", "topk_kernels.h", "plain_kernels.h")] + [
    os.path.join(os.path.dirname(HERE), "include", "comp_ams.h"),
    os.path.join(os.path.dirname(HERE), "include", "comp_ams_tuning.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                       # one rounding per operation, as in the definitions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


# A plain-C caller of the ABI (tests/c/abi_roundtrip.c), built next to the library so that the GPU tests can run it:
# gcc, the HIP runtime API header for device memory, the library by its path.
C_CALLER_SRC = os.path.join(os.path.dirname(HERE), "tests", "c", "abi_roundtrip.c")
C_CALLER = os.path.join(os.path.dirname(HERE), "tests", "c", "abi_roundtrip.bin")


def build_c_caller(verbose: bool = False) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-I", os.path.join(os.path.dirname(HERE), "include"),
           "-I", os.path.join(rocm, "include"), "-o", C_CALLER, C_CALLER_SRC, "-L", HERE, "-lcomp_ams",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2111_00705_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_CALLER


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB] + SOURCES
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        build_c_caller(verbose)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
