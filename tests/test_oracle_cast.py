"""Pins for the oracle's cast-copy: closed forms, numpy on the special cases where numpy's
definition is the same, and the exact-rational brute force over every dtype pair."""
import itertools
import math

import numpy as np
import pytest

import brute
import exactmath as X
from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import DTYPES, View

INT_TYPES = X.SIGNED + X.UNSIGNED


def _cast(src: View, dst_dtype: str) -> np.ndarray:
    dst = View.empty(dst_dtype, src.sizes)
    O.cast_copy(src, dst)
    return dst.to_numpy()


EDGE = np.array([0.0, -0.0, 0.999999, -0.999999, 1.5, -1.5, 2.5, -2.5, 127.0, 127.9, 128.0, -128.0,
                 -128.9, -129.0, 255.0, 255.9, 256.0, 32767.0, 32767.5, 32768.0, 32768.5, -32768.0,
                 -32768.5, -32769.0, 65535.9, 65536.0, 2147483647.0, 2147483647.5, 2147483648.0,
                 -2147483648.0, -2147483649.0, 4294967295.0, 4294967296.0, 9.2233720368547748e18,
                 9.223372036854775807e18, -9.223372036854775808e18, -9.3e18, 1.8446744073709550e19,
                 1.8446744073709552e19, 1e300, -1e300, math.inf, -math.inf, math.nan, 5e-324,
                 -5e-324, 1e-310], dtype=np.float64)


@pytest.mark.parametrize("dst", INT_TYPES)
def test_double_to_int_closed_form(dst):
    """clamp(trunc(x), lo, hi), NaN -> 0: evaluated here with Python's exact integers."""
    lo, hi = X.int_range(dst)
    got = _cast(View.from_numpy(EDGE), dst)
    for x, g in zip(EDGE, got):
        if math.isnan(x):
            want = 0
        elif math.isinf(x):
            want = hi if x > 0 else lo
        else:
            want = min(max(math.trunc(x), lo), hi)
        assert int(g) == want, (x, dst, int(g), want)


def test_config2_rule_values():
    """The stated rule for double -> int16: toward zero, saturating to [-32768, 32767], NaN -> 0."""
    x = np.array([1.9, -1.9, 32767.4, 32767.9, 32768.0, 4e4, -32768.9, -32769.0, -4e4, math.nan, 0.5, -0.5])
    want = np.array([1, -1, 32767, 32767, 32767, 32767, -32768, -32768, -32768, 0, 0, 0], dtype=np.int16)
    assert np.array_equal(_cast(View.from_numpy(x), "int16"), want)


@pytest.mark.parametrize("src", ("half", "float"))
@pytest.mark.parametrize("dst", INT_TYPES)
def test_narrow_float_to_int_equals_double_route(src, dst):
    """half/float -> double is exact, so casting through double must give the same integers."""
    rng = rng_for(21)
    v = random_view(rng, src, (400,))
    wide = View.from_numpy(v.to_numpy().astype(np.float64))
    assert np.array_equal(_cast(v, dst), _cast(wide, dst))


@pytest.mark.parametrize("src,dst", [(s, d) for s in ("bool",) + INT_TYPES for d in INT_TYPES])
def test_int_to_int_saturates(src, dst):
    rng = rng_for(22)
    v = random_view(rng, src, (300,))
    lo, hi = X.int_range(dst)
    vals = [int(t) for t in v.to_numpy().reshape(-1)]
    want = [min(max(t, lo), hi) for t in vals]
    assert [int(t) for t in _cast(v, dst)] == want


@pytest.mark.parametrize("src,dst", [(s, d) for s in ("bool",) + INT_TYPES + X.REAL for d in X.REAL])
def test_to_float_matches_numpy_round_to_nearest_even(src, dst):
    """numpy's astype to a floating type rounds to nearest even in one step: same definition."""
    rng = rng_for(23)
    v = random_view(rng, src, (2000,))
    a = v.to_numpy()
    with np.errstate(over="ignore", invalid="ignore"):
        want = a.astype(DTYPES[dst][1])
    got = _cast(v, dst)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    u = {2: np.uint16, 4: np.uint32, 8: np.uint64}[want.itemsize]
    assert np.array_equal(got[~nan].view(u), want[~nan].view(u))


def test_int64_to_float_hard_cases():
    # values needing a single rounding from 64 bits to 24: midpoints and their neighbours
    xs = []
    for e in (24, 25, 40, 62):
        base = 1 << e
        ulp = 1 << (e - 23)
        for k in (1, 3, 5):
            mid = base + k * ulp // 2
            xs += [mid - 1, mid, mid + 1, -(mid - 1), -mid, -(mid + 1)]
    xs += [2 ** 63 - 1, -2 ** 63, 2 ** 53 + 1, 2 ** 53 + 3]
    a = np.array(xs, dtype=np.int64)
    got = _cast(View.from_numpy(a), "float")
    from fractions import Fraction
    want = [X.round_fraction(Fraction(int(t)), "float") for t in a]
    assert [float(g) for g in got] == want
    ua = np.array([2 ** 64 - 1, 2 ** 64 - 2 ** 39, 2 ** 64 - 2 ** 40 - 2 ** 39, 2 ** 63 + 2 ** 39 + 1], dtype=np.uint64)
    got = _cast(View.from_numpy(ua), "float")
    assert [float(g) for g in got] == [X.round_fraction(Fraction(int(t)), "float") for t in ua]
    got = _cast(View.from_numpy(ua), "double")
    assert [float(g) for g in got] == [X.round_fraction(Fraction(int(t)), "double") for t in ua]


def test_to_bool_and_from_bool():
    x = np.array([0.0, -0.0, 1e-320, math.nan, -3.0, math.inf])
    assert list(_cast(View.from_numpy(x), "bool")) == [False, False, True, True, True, True]
    z = np.array([0 + 0j, 0 + 1j, 1 + 0j, complex(0.0, math.nan), complex(-0.0, -0.0)])
    assert list(_cast(View.from_numpy(z), "bool")) == [False, True, True, True, False]
    b = np.array([True, False])
    for dst in INT_TYPES + X.REAL:
        assert [float(t) for t in _cast(View.from_numpy(b), dst)] == [1.0, 0.0]
    g = _cast(View.from_numpy(b), "cdouble")
    assert list(g) == [1 + 0j, 0 + 0j]
    # a stored bool byte other than 0/1 still reads as true
    raw = View(np.array([0, 1, 2, 255], dtype=np.uint8), "bool", (4,), (1,), 0)
    assert list(_cast(raw, "int32")) == [0, 1, 1, 1]


def test_complex_real_conversions():
    z = np.array([1.5 - 2.5j, -0.0 + 7j, complex(math.inf, 1.0)], dtype=np.complex128)
    assert list(_cast(View.from_numpy(z), "double")) == [1.5, -0.0, math.inf]   # real part
    assert list(_cast(View.from_numpy(z), "int8")) == [1, 0, 127]
    r = np.array([1.25, -3.0], dtype=np.float32)
    g = _cast(View.from_numpy(r), "cfloat")
    assert list(g) == [1.25 + 0j, -3 + 0j]
    assert not np.signbit(g.imag).any()                                         # imaginary part is +0
    # the imaginary part of a complex double tensor is a double view on the same storage
    zz = View.from_numpy(z)
    imag = View(zz.storage, "double", zz.sizes, zz.strides, zz.offset + 8)
    assert list(_cast(imag, "double")) == [-2.5, 7.0, 1.0]


@pytest.mark.parametrize("src,dst", list(itertools.product(X.ALL, X.ALL)))
def test_every_pair_against_exact_rational_brute_force(src, dst):
    rng = rng_for(3000 + 15 * X.ALL.index(src) + X.ALL.index(dst))
    base = random_view(rng, src, (3, 4, 5))
    v = base.permute(2, 0, 1).slice(0, 0, 5, 2).flip(1)      # strided, reversed, permuted
    out = View.empty(dst, v.sizes, order="F")
    want = brute.unary("ident", v, out)
    O.cast_copy(v, out)
    assert brute.storages_match(dst, out.storage, want, out)


def test_config2_distribution_against_numpy_clip():
    """On N(0, 2e4) data the rule equals clip-then-truncate done by numpy on finite values."""
    rng = rng_for(24)
    x = rng.standard_normal(20000) * 2e4
    x[rng.random(20000) < 1e-3] = math.nan
    got = _cast(View.from_numpy(x), "int16")
    want = np.where(np.isnan(x), 0, np.trunc(np.clip(np.nan_to_num(x), -32768, 32767))).astype(np.int16)
    assert np.array_equal(got, want)
    assert (got == 32767).sum() > 100 and (got == -32768).sum() > 100  # saturation really occurs
