"""Pins for the oracle's reduce-of-an-elementwise-result (inner products, norms, counts of a
comparison): exact integer and rational arithmetic on small inputs, explicit replication for
broadcast operands, and the cases that reduce to a NumPy routine."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import exactmath as X
from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import View


def _run(ew, red, a, b, axes, out_dtype, mid):
    shape = np.broadcast_shapes(tuple(a.sizes), tuple(b.sizes))
    kept = [s for d, s in enumerate(shape) if d not in axes]
    out = View.empty(out_dtype, kept)
    O.binary_reduce(ew, red, a, b, list(axes), out, mid)
    return out.to_numpy()


@pytest.mark.parametrize("dt", ("int8", "int32", "int64", "uint16"))
def test_integer_inner_product_is_exact(dt):
    rng = rng_for(8100 + X.ALL.index(dt))
    a = random_view(rng, dt, (7, 33)).flip(1)
    b = random_view(rng, dt, (33, 7)).permute(1, 0)
    acc = "uint64" if dt in X.UNSIGNED else "int64"
    got = _run("mul", "sum", a, b, (1,), acc, dt)
    x, y = a.to_numpy(), b.to_numpy()
    lo, hi = X.int_range(dt)
    width = hi - lo + 1
    for r in range(7):
        # each product wraps to the element type first (the intermediate tensor has that type)
        total = 0
        for k in range(33):
            p = (int(x[r, k]) * int(y[r, k]) - lo) % width + lo
            total += p
        total &= (1 << 64) - 1
        if acc == "int64" and total >> 63:
            total -= 1 << 64
        assert int(got[r]) == total


def test_float_inner_product_within_the_rounding_bound():
    rng = rng_for(8110)
    a = random_view(rng, "float", (5, 2000), specials=False)
    b = random_view(rng, "float", (5, 2000), specials=False)
    got = _run("mul", "sum", a, b, (1,), "double", "float")
    x, y = a.to_numpy(), b.to_numpy()
    prod = (x * y).astype(np.float32)            # one IEEE single rounding per product
    for r in range(5):
        if not np.all(np.isfinite(prod[r])):
            continue
        exact = math.fsum(float(t) for t in prod[r])
        mag = math.fsum(abs(float(t)) for t in prod[r])
        assert abs(float(got[r]) - exact) <= 2.0 ** -52 * 2000 * mag + 1e-300


def test_squared_norm_of_small_integers_in_floating_point_is_exact():
    # values small enough that every product and partial sum is exact in single precision
    rng = rng_for(8111)
    v = rng.integers(-30, 31, size=(6, 50)).astype(np.float32)
    a = View.from_numpy(v)
    got = _run("mul", "sum", a, a.fresh_copy(), (1,), "float", "float")
    assert np.array_equal(got, (v.astype(np.int64) ** 2).sum(axis=1).astype(np.float32))


def test_count_of_complex_magnitude_comparison_matches_exact_rationals():
    rng = rng_for(8112)
    a = random_view(rng, "cfloat", (4, 60), specials=False)
    b = random_view(rng, "cfloat", (4, 60), specials=False)
    got = _run("absgt", "sum", a, b, (0, 1), "int64", "bool")
    za, zb = a.to_numpy(), b.to_numpy()
    count = 0
    for p, q in zip(za.reshape(-1), zb.reshape(-1)):
        ma = Fraction(float(p.real)) ** 2 + Fraction(float(p.imag)) ** 2
        mb = Fraction(float(q.real)) ** 2 + Fraction(float(q.imag)) ** 2
        if not (math.isfinite(p.real) and math.isfinite(p.imag) and math.isfinite(q.real) and math.isfinite(q.imag)):
            continue
        # the mask compares the double-rounded squared magnitudes; exact comparison agrees
        # unless the two differ by less than one part in 2^52
        if ma != mb and abs(ma - mb) <= max(ma, mb) * Fraction(1, 2 ** 52):
            pytest.skip("near tie in the random data")
        count += ma > mb
    assert int(got) == count


def test_any_all_of_comparisons_and_numpy_agreement():
    rng = rng_for(8113)
    a = random_view(rng, "int32", (9, 11))
    b = random_view(rng, "int32", (9, 11))
    x, y = a.to_numpy(), b.to_numpy()
    assert np.array_equal(_run("lt", "any", a, b, (1,), "bool", "bool"), (x < y).any(axis=1))
    assert np.array_equal(_run("ge", "all", a, b, (0,), "bool", "bool"), (x >= y).all(axis=0))
    assert np.array_equal(_run("eq", "sum", a, a.fresh_copy(), (0, 1), "int64", "bool"), np.int64(99))
    f = random_view(rng, "double", (8, 13), specials=False)
    g = random_view(rng, "double", (8, 13), specials=False)
    assert np.array_equal(_run("max", "min", f, g, (1,), "double", "double"),
                          np.maximum(f.to_numpy(), g.to_numpy()).min(axis=1))


def test_broadcast_operand_equals_explicit_replication():
    rng = rng_for(8114)
    a = random_view(rng, "double", (6, 5, 7), specials=False)
    row = random_view(rng, "double", (7,), specials=False)
    col = random_view(rng, "double", (5, 1), specials=False)
    for b in (row, col):
        full = View.from_numpy(np.ascontiguousarray(np.broadcast_to(b.to_numpy(), (6, 5, 7))))
        for axes in [(2,), (0,), (0, 1, 2), (1, 2)]:
            assert np.array_equal(_run("sub", "sum", a, b, axes, "double", "double"),
                                  _run("sub", "sum", a, full, axes, "double", "double"))


def test_intermediate_type_matters():
    # products that overflow half precision become infinite in a half intermediate, not in a float one
    a = View.from_numpy(np.full((4,), 300.0, dtype=np.float16))
    assert np.isinf(_run("mul", "sum", a, a.fresh_copy(), (0,), "float", "half"))
    wide = View.from_numpy(np.full((4,), 300.0, dtype=np.float32))
    assert float(_run("mul", "sum", wide, wide.fresh_copy(), (0,), "float", "float")) == 360000.0
