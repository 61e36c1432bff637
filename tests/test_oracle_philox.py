"""Pins for the oracle's Philox-4x32-10 (the random source of the stochastic
rounding; the paper only says the number is generated on the fly, App. A.1)."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
from tests import pymodel


def test_agrees_with_independent_python_implementation():
    rng = np.random.default_rng(0)
    for _ in range(20000):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64).astype(np.uint32)
        assert tuple(int(v) for v in oracle.philox4x32_10(ctr, key)) == pymodel.philox4x32_10(
            tuple(int(v) for v in ctr), tuple(int(v) for v in key))


def test_element_keying():
    """Element i of stream s under seed k reads word i mod 4 of the block whose
    counter is (i / 4, s) and whose key is k (both as little-endian 32-bit halves)."""
    for seed, sid, i in [(0, 0, 0), (1, 2, 3), (2**40 + 7, (5 << 8) | 2, 2**34 + 1), (2**64 - 1, 2**64 - 1, 2**40 - 1)]:
        blk = i // 4
        words = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, sid & 0xFFFFFFFF, sid >> 32],
                                     [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.random_word(seed, sid, i) == int(words[i % 4])
        assert oracle.random_word(seed, sid, i) == pymodel.random_word(seed, sid, i)


def test_counter_to_output_is_injective():
    key = np.array([123, 456], np.uint32)
    seen = set()
    n = 1 << 17
    for c in range(n):
        out = oracle.philox4x32_10([c, 0, 0, 0], key)
        seen.add(out.tobytes())
    assert len(seen) == n


def test_top17_bits_are_uniform():
    n = 1 << 20
    r = np.fromiter((oracle.random_word(77, 3, i) >> 15 for i in range(n)), dtype=np.int64, count=n)
    assert r.min() >= 0 and r.max() < 2**17
    counts = np.bincount(r >> 9, minlength=256)            # 256 equal cells
    expected = n / 256
    chi2 = ((counts - expected) ** 2 / expected).sum()
    # chi-square with 255 dof: mean 255, sd 22.6
    assert chi2 < 255 + 5 * 22.6
    # neighbouring elements (words of one block, and of adjacent blocks) are uncorrelated
    a = r[:-1].astype(np.float64) - r.mean()
    b = r[1:].astype(np.float64) - r.mean()
    corr = (a * b).mean() / r.var()
    assert abs(corr) < 5 / np.sqrt(n)


@pytest.fixture(scope="module")
def rocrand_helper(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc) or not os.path.exists("/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"):
        pytest.skip("hipcc or the rocRAND header is not available")
    src = os.path.join(os.path.dirname(__file__), "helpers", "rocrand_philox_host.cpp")
    so = str(tmp_path_factory.mktemp("rr") / "librr.so")
    res = subprocess.run([hipcc, "-x", "hip", "--offload-arch=gfx950", "-O1", "-shared", "-fPIC", src, "-o", so],
                         capture_output=True, text=True)
    if res.returncode != 0:
        pytest.skip("could not build the rocRAND host helper: " + res.stderr[-300:])
    L = ctypes.CDLL(so)
    L.rocrand_philox_words.argtypes = [ctypes.c_ulonglong, ctypes.c_ulonglong, ctypes.c_ulonglong, ctypes.c_void_p,
                                       ctypes.c_int]
    L.rocrand_philox_words.restype = None
    return L


def test_same_stream_as_rocrand_philox(rocrand_helper):
    """Library pin: element i of (seed, stream) reads the i-th output of the
    standard Philox4x32-10 stream rocRAND produces for seed, subsequence = stream."""
    for seed, sid, start in [(0, 0, 0), (0x1234567890ABCDEF, 7, 5), (42, (3 << 8) | 1, 2**33 + 2)]:
        n = 64
        out = np.zeros(n, np.uint32)
        rocrand_helper.rocrand_philox_words(seed, sid, start, out.ctypes.data, n)
        mine = [oracle.random_word(seed, sid, start + j) for j in range(n)]
        assert mine == [int(v) for v in out]
