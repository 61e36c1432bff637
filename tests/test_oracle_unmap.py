"""Pins for the oracle's non-linear inverse mapping (Sec. 3.2, exponent sum of Sec. 3.3)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pymodel
from tests.test_oracle_map import read_golden


def test_paper_alignment_example():
    g = read_golden("sec3_2_alignment_example.txt")
    mant = int(g["in_mantissa"].replace(".", ""), 2)                 # 0101 -> 5
    frac_digits = len(g["in_mantissa"].split(".")[1])                # point after the first digit
    in_exp = int(g["in_exponent"])
    # integer mantissa 5 whose unit is 2^(127 - 3): pick eA so that lsb(eA) = in_exp - frac_digits
    eA = in_exp - frac_digits + 133
    out = oracle.unmap(np.array([mant], np.int32), eA, None)
    bits = int(out.view(np.uint32)[0])
    out_exp = int(g["out_exponent"])
    out_frac = int(g["out_mantissa"].split(".")[1], 2) << (23 - len(g["out_mantissa"].split(".")[1]))
    assert g["out_mantissa"].startswith("1.")                         # normalised: leading one
    assert bits == ((out_exp + 127) << 23) | out_frac
    assert float(out[0]) == 1.25 * 2.0 ** 125


def test_integers_up_to_2_pow_24_are_exact():
    step = 1 << 22
    for lo in range(-(1 << 24), (1 << 24) + 1, step):
        acc = np.arange(lo, min(lo + step, (1 << 24) + 1), dtype=np.int32)
        for eA, eB in ((133, 133), (140, 120)):
            out = oracle.unmap(acc, eA, eB)
            E = (eA - 133) + (eB - 133)
            assert np.array_equal(out.astype(np.float64), np.ldexp(acc.astype(np.float64), E))


def test_exponent_is_the_sum_of_the_operand_exponents():
    acc = np.array([1, -3, 1000], np.int32)
    for eA in (1, 100, 133, 254):
        for eB in (1, 90, 133, 254):
            E = (eA - 133) + (eB - 133)
            want = [pymodel.round_to_f32(Fraction(int(a)) * pymodel.pow2(E)) for a in acc]
            got = oracle.unmap(acc, eA, eB).view(np.uint32).tolist()
            assert got == want, (eA, eB)


def test_single_rounding_ties_to_even_subnormals_and_overflow():
    acc = np.array([(1 << 24) + 1, (1 << 24) + 3, (1 << 25) + 2, (1 << 25) + 6, -(1 << 24) - 1, 2**31 - 1, -2**31,
                    (1 << 24) + 2, 0x00FFFFFF, 3, 1, -1, 0], dtype=np.int64).astype(np.int32)
    rng = np.random.default_rng(0)
    acc = np.concatenate([acc, rng.integers(-2**31, 2**31, 500, dtype=np.int64).astype(np.int32)])
    # E from deep sub-normal results through normal to overflow
    for eA, eB in [(1, 1), (1, 90), (1, 100), (10, 100), (60, 66), (133, 133), (254, 200), (254, 240), (254, 254)]:
        E = (eA - 133) + (eB - 133)
        want = [pymodel.round_to_f32(Fraction(int(a)) * pymodel.pow2(E)) for a in acc]
        got = oracle.unmap(acc, eA, eB).view(np.uint32).tolist()
        assert got == want, (eA, eB)
    assert oracle.unmap(np.array([(1 << 24) + 1], np.int32), 133, 133)[0] == float(1 << 24)       # tie -> even
    assert oracle.unmap(np.array([(1 << 24) + 3], np.int32), 133, 133)[0] == float((1 << 24) + 4)
    assert np.isinf(oracle.unmap(np.array([1 << 30], np.int32), 254, 254)[0])
    assert oracle.unmap(np.array([0], np.int32), 254, 254).view(np.uint32)[0] == 0                  # +0.0


def test_sums_wider_than_32_bits_are_rounded_once():
    """int64 sums (contractions beyond 133144 terms): against the exact rational model, ties and all, from
    sub-normal results to overflow; and equal to the int32 path wherever a value fits both."""
    rng = np.random.default_rng(3)
    acc = np.array([(1 << 40) + (1 << 16), (1 << 40) + 3 * (1 << 16), -(1 << 40) - (1 << 16), (1 << 33) + (1 << 9),
                    (1 << 33) + (1 << 9) + 1, (1 << 33) + (1 << 9) - 1, 2**31, -2**31 - 1, 16129 * 2**31 - 1,
                    -(16129 * 2**31 - 1), 1, -1, 0], dtype=np.int64)
    acc = np.concatenate([acc, rng.integers(-2**46, 2**46, 400, dtype=np.int64), rng.integers(-2**33, 2**33, 100, dtype=np.int64)])
    for eA, eB in [(1, 1), (1, 90), (10, 100), (60, 66), (133, 133), (200, 200), (254, 230), (254, 254)]:
        E = (eA - 133) + (eB - 133)
        want = [pymodel.round_to_f32(Fraction(int(a)) * pymodel.pow2(E)) for a in acc]
        got = oracle.unmap(acc, eA, eB).view(np.uint32).tolist()
        assert got == want, (eA, eB)
    assert oracle.unmap(np.array([(1 << 40) + (1 << 16)], np.int64), 133, 133)[0] == float(1 << 40)        # tie -> even
    small = rng.integers(-2**31, 2**31, 300, dtype=np.int64)
    assert np.array_equal(oracle.unmap(small, 120, 131).view(np.uint32), oracle.unmap(small.astype(np.int32), 120, 131).view(np.uint32))


def test_lower_bit_widths_change_only_the_unit():
    acc = np.array([5, -9], np.int32)
    for bits in (8, 7, 6, 5, 4):
        out = oracle.unmap(acc, 127, 127, bitsA=bits, bitsB=8)
        assert np.array_equal(out, acc * 2.0 ** (-(bits - 2)) * 2.0 ** -6)


def test_unmap_i8_is_exact():
    q = np.arange(-128, 128, dtype=np.int16).astype(np.int8)
    out = oracle.unmap_i8(q, 127 + 3)
    assert np.array_equal(out, q.astype(np.float32) * np.float32(2.0 ** (3 - 6)))
