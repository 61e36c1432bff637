"""Compile the CPU oracle (oracle/fxp_ref.cpp) into oracle/libfxp_ref.so.

The oracle is test infrastructure: tests, the smoke check and the benchmark's
cpu_baseline leg load it; the product never does.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fxp_ref.cpp")
LIB = os.path.join(HERE, "libfxp_ref.so")


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-Wall", "-Wextra",
           SRC, "-o", LIB + ".tmp"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
