"""Compile oracle/difa_oracle.c into oracle/libdifa_oracle.so (gcc + OpenMP, host only).

Test infrastructure: building the checker is not using it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "difa_oracle.c")
LIB = os.path.join(HERE, "libdifa_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # x86-64-v3 (AVX2+FMA) rather than -march=native: the library is built in one
    # container and run on another host.
    cmd = ["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
