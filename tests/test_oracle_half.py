"""Pins for the oracle's half-precision conversions (IEEE 754 binary16).

Independent references: numpy's float16 (a library routine with the same definition) over the
whole 16-bit pattern space, and an exact-rational rounding written out in tests/exactmath.py.
"""
import math
from fractions import Fraction

import numpy as np

import exactmath as X
from oracle import binding as O


def test_decode_all_patterns_matches_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_bits_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint64), want[~nan].view(np.uint64))  # incl. sign of zero


def test_roundtrip_identity_all_non_nan_patterns():
    for b in range(65536):
        d = O.half_bits_to_double(b)
        if math.isnan(d):
            assert math.isnan(O.half_bits_to_double(O.double_to_half_bits(d)))
        else:
            assert O.double_to_half_bits(d) == b


def test_encode_random_doubles_matches_numpy():
    rng = np.random.Generator(np.random.PCG64(11))
    x = np.concatenate([
        rng.standard_normal(100000),
        rng.standard_normal(100000) * 1e4,
        np.ldexp(rng.standard_normal(100000), rng.integers(-30, 18, size=100000)),
    ])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([O.double_to_half_bits(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_encode_midpoints_tie_to_even_and_neighbours():
    # every midpoint between consecutive non-negative halfs, and the doubles just beside it
    for b in range(0, 0x7C00):
        lo = Fraction(O.half_bits_to_double(b))
        hi_val = O.half_bits_to_double(b + 1)
        hi = Fraction(2) ** 16 if math.isinf(hi_val) else Fraction(hi_val)
        mid = float((lo + hi) / 2)  # exact in double
        even = b if b % 2 == 0 else b + 1
        assert O.double_to_half_bits(mid) == even
        assert O.double_to_half_bits(-mid) == (even | 0x8000)
        assert O.double_to_half_bits(math.nextafter(mid, 0.0)) == b
        assert O.double_to_half_bits(math.nextafter(mid, math.inf)) == b + 1


def test_encode_against_exact_rational_rounding():
    rng = np.random.Generator(np.random.PCG64(12))
    xs = np.ldexp(rng.standard_normal(3000), rng.integers(-28, 17, size=3000))
    for v in xs:
        want = X.round_fraction(Fraction(float(v)), "half", float(v))
        got = O.half_bits_to_double(O.double_to_half_bits(float(v)))
        assert (math.isinf(want) and math.isinf(got) and (want > 0) == (got > 0)) or got == want
        assert math.copysign(1, got) == math.copysign(1, want)


def test_specials():
    assert O.double_to_half_bits(0.0) == 0x0000
    assert O.double_to_half_bits(-0.0) == 0x8000
    assert O.double_to_half_bits(math.inf) == 0x7C00
    assert O.double_to_half_bits(-math.inf) == 0xFC00
    assert O.double_to_half_bits(65504.0) == 0x7BFF
    assert O.double_to_half_bits(65519.99) == 0x7BFF
    assert O.double_to_half_bits(65520.0) == 0x7C00
    assert O.double_to_half_bits(1e300) == 0x7C00
    assert O.double_to_half_bits(2.0 ** -24) == 0x0001
    assert O.double_to_half_bits(2.0 ** -25) == 0x0000          # tie -> even (zero)
    assert O.double_to_half_bits(math.nextafter(2.0 ** -25, 1)) == 0x0001
    h = O.double_to_half_bits(math.nan)
    assert (h & 0x7C00) == 0x7C00 and (h & 0x3FF) != 0
