"""Builds ``libef21.so`` (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libef21.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",                                     # hardware fp32 atomic add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
    "-Wall", "-Wno-unused-command-line-argument", "-parallel-jobs=8",
]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False) -> str:
    """Compile every .hip source into paper_2106_05203_amd/libef21.so. Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


C_CLIENT_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_client.c")
C_CLIENT = os.path.join(os.path.dirname(HERE), "tests", "c_client")


def build_c_client(verbose: bool = False) -> str:
    """Compile tests/c_client.c, a client of the library written in plain C, with gcc (the host compiler: the
    client holds no device code) against include/ef21.h, libef21.so and the HIP runtime.  The library is found
    at run time relative to the executable."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(os.path.dirname(HERE), "include"), "-I", os.path.join(rocm, "include"),
           C_CLIENT_SRC, "-o", C_CLIENT, "-L", HERE, "-lef21", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2106_05203_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"),
           "-Wl,-rpath-link," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return C_CLIENT


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_client(verbose=True))
