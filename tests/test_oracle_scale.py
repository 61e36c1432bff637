"""Pins for the oracle's scale (Sec. 3.1: e_max = max of the exponents)."""
import math

import numpy as np
import pytest

import oracle


def brute_scale(x):
    """max over elements of ilogb(|x|) + 127 via the C library's frexp; zeros
    and sub-normals weigh as the smallest normal binade (field value 1)."""
    best = 1
    for v in np.asarray(x, dtype=np.float32).ravel().tolist():
        if v == 0.0:
            continue
        if math.isinf(v) or math.isnan(v):
            best = max(best, 255)
            continue
        m, ex = math.frexp(abs(v))       # |v| = m * 2^ex, m in [0.5, 1)
        best = max(best, max(1, (ex - 1) + 127))
    return best


@pytest.mark.parametrize("seed", range(4))
def test_matches_frexp_bruteforce(seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(5000) * 10.0 ** rng.uniform(-30, 30)).astype(np.float32)
    assert oracle.scale(x) == brute_scale(x)


def test_special_cases():
    assert oracle.scale(np.zeros(0, np.float32)) == 1
    assert oracle.scale(np.zeros(17, np.float32)) == 1
    assert oracle.scale(np.array([1.0], np.float32)) == 127
    assert oracle.scale(np.array([-1.0], np.float32)) == 127
    for k in (-126, -20, 0, 1, 64, 127):
        p = np.float32(2.0) ** np.float32(k)
        assert oracle.scale(np.array([0.1 * p, p], np.float32)) == k + 127
        below = np.nextafter(p, np.float32(0), dtype=np.float32)
        assert oracle.scale(np.array([below], np.float32)) == max(1, k - 1 + 127)
    sub = np.array([1e-45, -3e-39, 0.0], np.float32)          # sub-normals only
    assert oracle.scale(sub) == 1
    assert oracle.scale(np.array([1.0, np.inf], np.float32)) == 255
    assert oracle.scale(np.array([np.nan, 1.0], np.float32)) == 255
    assert oracle.scale(np.array([3.0, -1000.0, 5.0], np.float32)) == 127 + 9   # sign ignored


def test_position_of_max_is_irrelevant():
    rng = np.random.default_rng(7)
    x = rng.standard_normal(1000).astype(np.float32)
    for pos in (0, 499, 999):
        y = x.copy()
        y[pos] = 4096.5
        assert oracle.scale(y) == 127 + 12
