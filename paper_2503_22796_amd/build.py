"""Compile the HIP/C++ sources under csrc/ into paper_2503_22796_amd/libdifa.so for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdifa.so")
OBJ = os.path.join(HERE, "_build")
HOST_SOURCES = ["difa_api.cpp", "difa_worklist.cpp", "difa_solver.cpp"]
KERNEL_SOURCES = ["difa_kernels.hip", "difa_rse.hip", "difa_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]
# Kernel files only.  The host files check their arguments for NaN and must keep IEEE comparisons.
KERNEL_FLAGS = [
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # NaN tensor values are outside the contract; without this every fmaxf pays a canonicalising v_max
    "-fno-honor-nans",
]


def build(verbose: bool = False, extra=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    for src in HOST_SOURCES + KERNEL_SOURCES:
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        flags = COMMON + (KERNEL_FLAGS if src in KERNEL_SOURCES else []) + list(extra)
        cmd = [HIPCC] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
