"""Build libfxp.so (the HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2207_08822_amd.build            # always rebuilds
    python -m paper_2207_08822_amd.build --if-stale  # only when a source is newer

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is switched
off for all device code and fp32 denormals are kept (the inverse mapping must
round into the sub-normal range, not flush).
"""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfxp.so")
OBJ = os.path.join(HERE, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-flush-denormals-to-zero", "-Xclang",
         "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "fxp.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    res = subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
    return obj


def build(force=True):
    if not force and not stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, sources()))
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp"],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_ceilings():
    """Standalone hardware-ceiling microbenchmark (not part of libfxp.so)."""
    src = os.path.join(HERE, "ceilings", "fxp_ceilings.hip")
    exe = os.path.join(HERE, "ceilings", "fxp_ceilings")
    res = subprocess.run([HIPCC, *[f for f in FLAGS if f != "-fPIC"], src, "-o", exe], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on fxp_ceilings.hip:\n" + res.stderr)
    return exe


if __name__ == "__main__":
    if "--ceilings" in sys.argv:
        print(build_ceilings())
    else:
        print(build(force="--if-stale" not in sys.argv))
