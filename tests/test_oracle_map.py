"""Pins for the oracle's linear fixed-point mapping (Sec. 3.1, App. A.1)."""
import os

import numpy as np
import pytest

import oracle
from tests import pymodel

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = v
    return out


def binary_fixed(s):
    """'h.fff' -> integer made of all digits."""
    return int(s.replace(".", ""), 2)


def test_paper_worked_example_kept_and_dropped_bits():
    g = read_golden("sec3_1_rounding_example.txt")
    m_shift = binary_fixed(g["shifted_mantissa"])
    assert len(g["shifted_mantissa"].replace(".", "")) == 24
    lo, hi = binary_fixed(g["lower_result"]), binary_fixed(g["upper_result"])
    assert (lo, hi) == (22, 23)
    low17 = m_shift & 0x1FFFF
    # Build a tensor whose second element has exactly this shifted mantissa:
    # the leading one of m_shift sits 2 places below the hidden-bit position,
    # so the element's exponent is e_max - 2 and its own mantissa is m_shift << 2.
    d = 24 - m_shift.bit_length()
    assert d == 2
    e_max = 130
    x = np.float32(np.ldexp(float(m_shift << d), (e_max - d) - 150))
    n = 1_000_000
    t = np.full((1, n), x, dtype=np.float32)
    t[0, 0] = np.ldexp(1.0, e_max - 127)              # plants e_max
    assert oracle.scale(t) == e_max
    q = oracle.map(t, e_max, seed=11, stream_id=5)[0, 1:]
    assert set(np.unique(q).tolist()) == {lo, hi}
    p = low17 / 2.0 ** 17                               # App. A.1: (x - x1)/(x2 - x1)
    assert abs(p - 0.33325) < 1e-5
    ups = int((q == hi).sum())
    sigma = np.sqrt((n - 1) * p * (1 - p))
    assert abs(ups - (n - 1) * p) < 4.5 * sigma
    # negated input: mirrored outputs, same decisions (sign handled apart from magnitude)
    qn = oracle.map(-t, e_max, seed=11, stream_id=5)[0, 1:]
    assert np.array_equal(qn, -q)


@pytest.mark.parametrize("bits", [8, 7, 6, 5, 4])
@pytest.mark.parametrize("e_max", [1, 60, 127, 133, 200, 254])
def test_exact_round_trip_of_grid_values(bits, e_max):
    """Values already on the fixed-point grid map to themselves for every seed
    and the inverse mapping gives the input back bit for bit."""
    sat = (1 << (bits - 1)) - 1
    k = np.arange(-sat, sat + 1, dtype=np.int64)
    E = pymodel.lsb_exponent(e_max, bits)
    x = np.ldexp(k.astype(np.float64), E).astype(np.float32).reshape(1, -1)
    assert np.array_equal(np.ldexp(k.astype(np.float64), E), x[0].astype(np.float64))   # representable
    assert oracle.scale(x) == e_max
    for seed in (0, 1, 2**63 + 5):
        q = oracle.map(x, e_max, seed=seed, stream_id=seed ^ 3, bits=bits)
        assert np.array_equal(q[0].astype(np.int64), k)
        back = oracle.unmap_i8(q, e_max, bits=bits)
        assert np.array_equal(back.view(np.uint32) & 0x7FFFFFFF, x.view(np.uint32) & 0x7FFFFFFF)
        assert np.array_equal(back, x)


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_against_exact_rational_model(bits):
    """Every element equals the big-integer / Fraction model: floor of the exact
    quotient plus one iff the independent Philox word's top bits are below the
    truncated remainder."""
    rng = np.random.default_rng(bits)
    x = (rng.standard_normal((7, 13)) * np.exp(rng.uniform(-12, 3, (7, 13)))).astype(np.float32)
    x[2, 3] = 0.0
    x[4, 4] = -0.0
    x[1, 1] = 1e-42        # sub-normal input
    e_max = oracle.scale(x)
    seed, sid = 0xDEADBEEFCAFE, (9 << 8) | 2
    q = oracle.map(x, e_max, seed=seed, stream_id=sid, bits=bits)
    for r in range(7):
        for c in range(13):
            i = r * 13 + c
            assert int(q[r, c]) == pymodel.map_one(float(x[r, c]), e_max, seed, sid, i, bits), (r, c)


def test_bracketing_range_and_sign():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((64, 257)) * 10.0 ** rng.uniform(-6, 2, (64, 257))).astype(np.float32)
    e_max = oracle.scale(x)
    q = oracle.map(x, e_max, seed=1).astype(np.float64)
    t = x.astype(np.float64) / 2.0 ** (e_max - 133)          # exact: power-of-two division in fp64
    assert np.all(np.abs(q) <= 127)
    assert np.all((q == np.floor(t)) | (q == np.ceil(t)) | (np.abs(t) > 127))
    assert np.all(np.sign(q) * np.sign(t) >= 0)
    assert np.abs(q).max() >= 64                               # the max element fills the top bit


def test_saturation_at_127_never_128():
    # max element with all seven kept bits set and a non-zero remainder
    e_max = 127
    x = np.full((1, 4096), np.float32(1.9999999), dtype=np.float32)
    x[0, ::2] *= -1
    q = oracle.map(x, e_max, seed=5)
    assert np.all(np.abs(q.astype(np.int32)) == 127)


def test_scale_larger_or_smaller_than_the_tensor():
    x = np.array([[1.0, -1.5, 0.75, 3.0]], np.float32)
    # larger scale: values simply sit lower in the register
    q = oracle.map(x, 127 + 5, rounding=oracle.NEAREST)
    assert q.tolist() == [[2, -3, 2, 6]]            # 0.75*2 = 1.5 -> half up
    # smaller scale than an element needs: that element saturates
    q = oracle.map(x, 127, rounding=oracle.NEAREST)
    assert q.tolist() == [[64, -96, 48, 127]]
    # shift of 24 or more positions empties the register
    q = oracle.map(np.array([[1.0, 2.0 ** -24, -(2.0 ** -23)]], np.float32), 127 + 0, seed=3)
    assert q[0, 0] == 64 and q[0, 1] == 0
    tiny = np.full((1, 100000), 2.0 ** -17, np.float32)        # d = 17: register holds 2^6, below the cut
    tiny[0, 0] = 1.0
    qt = oracle.map(tiny, 127, seed=9)[0, 1:]
    assert set(np.unique(qt).tolist()) <= {0, 1}
    p = 64 * 2.0 ** -17 / 1.0                                  # |x| / LSB = 2^-17 / 2^-6 ... = 2^-11
    assert abs(p - 2.0 ** -11) < 1e-12
    assert abs(qt.mean() - p) < 4.5 * np.sqrt(p / qt.size)


def test_non_finite_inputs_are_defined():
    x = np.array([[np.inf, -np.inf, np.nan, 1.0, -2.0 ** 127]], np.float32)
    assert oracle.scale(x) == 255
    q = oracle.map(x, 255, seed=1)
    # Inf saturates, NaN gives 0, 1.0 is shifted out, 2^127 is 1.0 shifted right by one place
    assert q.tolist() == [[127, -127, 0, 0, -32]]


def test_subnormal_and_zero_tensors():
    z = np.zeros((3, 5), np.float32)
    assert np.all(oracle.map(z, oracle.scale(z)) == 0)
    sub = np.array([[2.0 ** -149 * 0x7FFFFF, -(2.0 ** -127), 2.0 ** -149]], np.float32)
    e = oracle.scale(sub)
    assert e == 1
    q = oracle.map(sub, e, rounding=oracle.NEAREST)
    # unit is 2^(1-133) = 2^-132; 0x7FFFFF * 2^-149 = (2^23-1) * 2^-17 units -> 64 (half up from 63.99)
    assert q.tolist() == [[64, -32, 0]]


def test_transposed_copy_is_identical():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((37, 52)).astype(np.float32)
    e = oracle.scale(x)
    q, qT = oracle.map(x, e, seed=4, stream_id=77, transposed=True)
    assert np.array_equal(q.T, qT)
    assert np.array_equal(q, oracle.map(x, e, seed=4, stream_id=77))


def test_determinism_and_stream_separation():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((64, 64)).astype(np.float32)
    e = oracle.scale(x)
    a = oracle.map(x, e, seed=1, stream_id=2)
    assert np.array_equal(a, oracle.map(x, e, seed=1, stream_id=2))
    assert not np.array_equal(a, oracle.map(x, e, seed=2, stream_id=2))
    assert not np.array_equal(a, oracle.map(x, e, seed=1, stream_id=3))
    # the element index, not the shape, selects the random word
    assert np.array_equal(a.ravel(), oracle.map(x.reshape(16, 256), e, seed=1, stream_id=2).ravel())


def test_monotone_for_a_fixed_random_word():
    xs = np.sort(np.random.default_rng(8).uniform(-3.9, 3.9, 2000).astype(np.float32))
    prev = -128
    for v in xs:
        t = np.array([[v, 4.0]], np.float32)
        q = int(oracle.map(t, 129, seed=21, stream_id=1)[0, 0])
        assert q >= prev
        prev = q


def _mean_error_z(x, e_max, q, bits=8):
    """z statistic of the summed rounding error in LSB units against the exact
    Bernoulli variance sum p(1-p), with p the exact fractional part."""
    t = np.abs(x.astype(np.float64)) / 2.0 ** (e_max - 127 - (bits - 2))
    frac = t - np.floor(t)
    delta = np.abs(q.astype(np.float64)) - t
    return delta.sum() / np.sqrt((frac * (1 - frac)).sum()), delta.mean()


def test_mean_rounding_error_is_zero_over_1e7_samples():
    rng = np.random.default_rng(0)
    n = 10_000_000
    x = rng.standard_normal(n, dtype=np.float32).reshape(2500, 4000)
    x[0, 0] = 8.0                      # power-of-two maximum: nothing reaches the saturating top code
    x = np.clip(x, -8.0, 8.0)
    e = oracle.scale(x)
    assert e == 130
    q = oracle.map(x, e, seed=2024, stream_id=1)
    z, mean = _mean_error_z(x, e, q)
    assert abs(z) < 4.0, (z, mean)
    # the truncating shift only costs < 2^-17 LSB per element, far below the noise floor
    assert abs(mean) < 1e-3


def test_nearest_rounding_fails_the_same_test_on_tiny_gradients():
    """Negative control: with round-to-nearest a tensor whose bulk is far below
    one unit loses its mean, which is the failure the paper's rounding avoids."""
    rng = np.random.default_rng(1)
    g = np.abs(rng.laplace(0, 1e-5, size=(1000, 1000))).astype(np.float32)
    g[0, 0] = 1.0
    e = oracle.scale(g)
    z_sr, _ = _mean_error_z(g, e, oracle.map(g, e, seed=3))
    z_rn, _ = _mean_error_z(g, e, oracle.map(g, e, rounding=oracle.NEAREST))
    assert abs(z_sr) < 4.0
    assert abs(z_rn) > 10.0


def test_row_slices_carry_the_index_of_the_whole_tensor():
    """map_rows on slices reassembles map of the whole tensor, and at element indices beyond 2^34 (counter words
    above the low one in use) every element equals the independent rational model with the same index."""
    rng = np.random.default_rng(12)
    x = rng.standard_normal((37, 24)).astype(np.float32)
    e = oracle.scale(x)
    whole = oracle.map(x, e, seed=9, stream_id=77)
    parts = [oracle.map_rows(x[a:b], a, e, seed=9, stream_id=77) for a, b in ((0, 5), (5, 6), (6, 37))]
    assert np.array_equal(np.concatenate(parts), whole)
    assert oracle.map_rows(x[:0], 3, e).shape == (0, 24)
    row0 = (1 << 34) // 24 + 12345                      # first element index above 2^34
    q = oracle.map_rows(x[:3], row0, e, seed=9, stream_id=77)
    for r in range(3):
        for c in range(24):
            i = (row0 + r) * 24 + c
            assert i >> 34 and int(q[r, c]) == pymodel.map_one(float(x[r, c]), e, 9, 77, i)
    assert not np.array_equal(q, whole[:3])              # not the words of rows 0..2
