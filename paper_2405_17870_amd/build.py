"""Build ``libnezha_sim.so`` (HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnezha_sim.so")
SOURCES = [os.path.join(CSRC, "nz_host.hip"), os.path.join(CSRC, "nz_index.cpp"),
           os.path.join(CSRC, "nz_balance.cpp"), os.path.join(CSRC, "nz_validate.cpp"),
           os.path.join(CSRC, "nz_placement.cpp")]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build libnezha_sim.so")
    return exe


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-ffp-contract=off",
           # keep the compiler from forming packed-fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


C_DRIVER_SRC = os.path.join(ROOT, "tests", "c_abi_gpu_driver.cpp")
C_DRIVER = os.path.join(ROOT, "tests", "libc_abi_gpu_driver.so")


def build_c_driver(verbose: bool = False) -> str:
    """Compile the plain C++ caller of the C ABI that tests/test_gpu_c_abi.py runs on a GPU
    (host code only; it links the shared library and finds it next to the package)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall",
           "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), C_DRIVER_SRC,
           "-L", HERE, "-lnezha_sim", "-Wl,-rpath,$ORIGIN/../paper_2405_17870_amd", "-o", C_DRIVER]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_DRIVER


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_driver(verbose=True))
