"""Build libfef.so (the C-ABI verify-step library) in-tree with hipcc for gfx950.

    python -m paper_2605_14305_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfef.so")
SOURCES = ["fef_api.hip", "head_gemm.hip", "head_gemm_tiled256.hip", "head_gemm_stream.hip", "head_gemm_rowstream.hip",
           "verify_kernels.hip", "ce_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose=True, extra_flags=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


HARNESS_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "abi_harness.cpp")
HARNESS = os.path.join(HERE, "abi_harness")


def build_harness(verbose=True):
    """The C++ program that calls libfef.so through include/fef.h alone (run by the GPU tests)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-std=c++17", "-O1", "-Wall", "-I", os.path.join(os.path.dirname(HERE), "include"), HARNESS_SRC,
           "-L", HERE, "-lfef", "-Wl,-rpath,$ORIGIN", "-o", HARNESS]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return HARNESS


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
    build_harness()
