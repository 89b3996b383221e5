"""Build libfef.so (the C-ABI verify-step library) in-tree with hipcc for gfx950.

    python -m paper_2605_14305_amd.build
"""
import os
import re
import subprocess
import sys
import tempfile

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
    check_rowstream_isa(verbose)
    return LIB


def _vgprs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def check_rowstream_isa(verbose=True):
    """head_gemm_rowstream.hip loads W into registers by inline assembly and waits for the data by
    hand, so the compiler believes a loaded value exists from the load statement on.  That is sound
    as long as the compiler never copies such a value before its wait, i.e. as long as every
    multiply takes its W operand from the very registers a load statement wrote.  This compiles
    the file to assembly and checks exactly that for each instantiation; a compiler that starts
    to shuffle these registers fails the build instead of producing a kernel that reads stale data."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "rowstream.s")
        flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
        subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", os.path.join(CSRC, "head_gemm_rowstream.hip"), "-o", out],
                       check=True, stderr=subprocess.DEVNULL)
        lines = open(out).read().split("\n")
    kernels = [i for i, l in enumerate(lines) if re.match(r"^_Z\w*head_rowstream_kernel\w*:", l)]
    if not kernels:
        raise RuntimeError("check_rowstream_isa: no head_rowstream_kernel in the assembly")
    for start in kernels:
        end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
        ring, in_asm = set(), False
        for l in lines[start:end]:
            t = l.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            elif in_asm and t.startswith("global_load_dwordx4"):
                ring |= _vgprs(t.split(",")[0])
        n = 0
        for l in lines[start:end]:
            t = l.strip()
            if t.startswith("v_mfma"):
                a_operand = t.split(None, 1)[1].split(",")[1]
                n += 1
                if not _vgprs(a_operand) <= ring:
                    raise RuntimeError(f"check_rowstream_isa: {lines[start].split(':')[0]}: W operand of '{t}' is not "
                                       "a register written by a load statement (the compiler copied a value in flight)")
        if n == 0 or not ring:
            raise RuntimeError("check_rowstream_isa: no loads or multiplies found")
        if verbose:
            print(f"check_rowstream_isa: {lines[start].split(':')[0]}: {n} multiplies read {len(ring)} load registers directly",
                  flush=True)


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
