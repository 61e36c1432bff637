"""Independent pure-Python models used to pin the CPU oracle.

Nothing here is derived from oracle/ or from the HIP sources: the Philox
generator is written from the published description (Salmon et al., SC'11:
two 32x32->64 multiplies per round, ten rounds, Weyl-sequence key schedule),
and the fixed-point arithmetic is done on exact rationals / big integers from
the mathematical definition of the format (value = q * 2^E).
"""
import struct
from fractions import Fraction

MASK32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    c0, c1, c2, c3 = ctr
    k0, k1 = key
    for rnd in range(10):
        p0 = 0xD2511F53 * c0
        p1 = 0xCD9E8D57 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK32, p1 & MASK32, ((p0 >> 32) ^ c3 ^ k1) & MASK32, p0 & MASK32
        k0 = (k0 + 0x9E3779B9) & MASK32
        k1 = (k1 + 0xBB67AE85) & MASK32
    return c0, c1, c2, c3


def random_word(seed, stream_id, i):
    blk = i // 4
    out = philox4x32_10((blk & MASK32, blk >> 32, stream_id & MASK32, stream_id >> 32), (seed & MASK32, seed >> 32))
    return out[i % 4]


def f32_bits(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def bits_f32(b):
    return struct.unpack("<f", struct.pack("<I", b))[0]


def exact_value(x):
    """fp32 value as an exact Fraction (finite inputs)."""
    return Fraction(float(x))


def lsb_exponent(e_max, bits=8):
    return e_max - 127 - (bits - 2)


def pow2(E):
    return Fraction(2) ** E


def floor_and_prob(x, e_max, bits=8):
    """Exact floor(|x| / 2^E) and the paper's round-up probability for |x|.

    The shift by d = e_max - e drops mantissa bits below bit 0 of the 24-bit
    register, so the compared remainder is the exact remainder truncated to a
    multiple of 2^-cut of one unit: P(up) = floor(frac * 2^cut) / 2^cut.
    """
    cut = 24 - (bits - 1)
    t = abs(exact_value(x)) / pow2(lsb_exponent(e_max, bits))
    fl = t.numerator // t.denominator
    frac = t - fl
    low = (frac * (1 << cut)).numerator // (frac * (1 << cut)).denominator
    return fl, low, cut


def map_one(x, e_max, seed, stream_id, i, bits=8):
    """Stochastically rounded fixed-point value of a finite x with |x| < 2^(e_max-126)."""
    fl, low, cut = floor_and_prob(x, e_max, bits)
    r = random_word(seed, stream_id, i) >> (32 - cut)
    q = fl + (1 if r < low else 0)
    q = min(q, (1 << (bits - 1)) - 1)
    return -q if (f32_bits(x) >> 31) else q


def round_to_f32(value):
    """Round an exact Fraction to the nearest fp32 (ties to even, gradual
    underflow, overflow to infinity) with integer arithmetic only; returns bits."""
    if value == 0:
        return 0
    sign = 0x80000000 if value < 0 else 0
    v = abs(value)
    # find e with 2^e <= v < 2^(e+1)
    e = v.numerator.bit_length() - v.denominator.bit_length()
    if pow2(e) > v:
        e -= 1
    if pow2(e + 1) <= v:
        e += 1
    e_q = max(e, -126)                 # exponent of the binade used for quantisation
    ulp = pow2(e_q - 23)
    n = v / ulp                        # number of ulps (>= 2^23 if normal)
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    # fl ulps of 2^(e_q-23); renormalise if it carried to 2^24
    if fl >= (1 << 24):
        fl >>= 1
        e_q += 1
    if fl >= (1 << 23):                # normal
        if e_q > 127:
            return sign | 0x7F800000
        return sign | ((e_q + 127) << 23) | (fl - (1 << 23))
    return sign | fl                   # sub-normal (or zero after rounding)
