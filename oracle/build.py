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
LIB_SAN = os.path.join(HERE, "libfxp_ref_san.so")      # the same source under AddressSanitizer + UBSan (host only)


def build(force=True, sanitize=False):
    """sanitize: build libfxp_ref_san.so instead, instrumented for out-of-bounds / use-after-free accesses and
    undefined behaviour (signed overflow, bad shifts, misaligned access); a finding ends the process.  A process
    that loads it must have the sanitizer runtime loaded first (see sanitizer_runtime())."""
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
           if sanitize else ["-O2"])
    cmd = ["g++", "-std=c++17", *opt, "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-Wall", "-Wextra",
           SRC, "-o", lib + ".tmp"]
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)
    return lib


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime the sanitized build needs in front of every other library
    (LD_PRELOAD of the process that loads it)."""
    out = subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    return os.path.realpath(out)


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv, sanitize="--sanitize" in sys.argv))
