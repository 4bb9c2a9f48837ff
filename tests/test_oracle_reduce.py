"""Pins for the oracle's axis and full reductions: exact integer sums, exactly rounded float
sums (math.fsum), numpy min/max on NaN-free data, invariants, and edge cases."""
import itertools
import math

import numpy as np
import pytest

import exactmath as X
from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import DTYPES, View


def _reduce(op, a: View, axes, out_dtype) -> np.ndarray:
    kept = [s for d, s in enumerate(a.sizes) if d not in axes]
    out = View.empty(out_dtype, kept)
    O.reduce(op, a, axes, out)
    return out.to_numpy()


@pytest.mark.parametrize("dt", ("bool",) + X.SIGNED + X.UNSIGNED)
@pytest.mark.parametrize("axes", [(0,), (1,), (2,), (0, 2), (1, 2), (0, 1, 2), (2, 0)])
def test_integer_sum_is_the_exact_sum(dt, axes):
    rng = rng_for(51)
    a = random_view(rng, dt, (5, 6, 7)).permute(1, 2, 0).flip(1)      # shape (6, 7, 5)
    arr = a.to_numpy()
    acc = "uint64" if dt in X.UNSIGNED else "int64"
    got = _reduce("sum", a, list(axes), acc)
    kept = [d for d in range(3) if d not in axes]
    for idx in itertools.product(*[range(arr.shape[d]) for d in kept]):
        sl = [slice(None)] * 3
        for d, i in zip(kept, idx):
            sl[d] = i
        exact = sum(int(t) for t in arr[tuple(sl)].reshape(-1))
        exact &= (1 << 64) - 1                                         # 64-bit wrap
        if acc == "int64" and exact >> 63:
            exact -= 1 << 64
        assert int(got[idx]) == exact


def test_int8_full_sum_closed_form_and_bound():
    rng = rng_for(52)
    x = rng.integers(-128, 127, size=100003, endpoint=True).astype(np.int8)
    got = _reduce("sum", View.from_numpy(x), [0], "int64")
    assert int(got) == sum(int(t) for t in x)
    assert abs(int(got)) <= x.size * 128
    # permutation independent
    got2 = _reduce("sum", View.from_numpy(rng.permutation(x)), [0], "int64")
    assert int(got2) == int(got)
    # extreme: all -128
    y = np.full(70000, -128, dtype=np.int8)
    assert int(_reduce("sum", View.from_numpy(y), [0], "int64")) == -128 * 70000


@pytest.mark.parametrize("dt,axis", [("float", 0), ("float", 1), ("half", 1), ("double", 0), ("double", 1)])
def test_float_sum_within_stated_bound_of_exact_sum(dt, axis):
    rng = rng_for(53)
    n0, n1 = 300, 2000
    x = rng.standard_normal((n0, n1)).astype(DTYPES[dt][1])
    a = View.from_numpy(x)
    got = _reduce("sum", a, [axis], "double")
    xs = x.astype(np.float64)
    lines = xs if axis == 1 else xs.T
    n = lines.shape[1]
    for i, line in enumerate(lines):
        exact = math.fsum(line)                    # correctly rounded exact sum
        bound = 2.0 ** -52 * n * float(np.abs(line).sum())
        assert abs(float(got[i]) - exact) <= bound
    if dt == "double":
        # compensated summation: essentially exact
        for i, line in enumerate(lines):
            assert abs(float(got[i]) - math.fsum(line)) <= 4 * 2.0 ** -53 * abs(math.fsum(line)) + 1e-300


def test_float_sum_is_rounded_once_to_the_output_type():
    rng = rng_for(54)
    x = rng.standard_normal((64, 999)).astype(np.float32)
    a = View.from_numpy(x)
    wide = _reduce("sum", a, [1], "double")
    narrow = _reduce("sum", a, [1], "float")
    assert np.array_equal(narrow, wide.astype(np.float32))
    # sequential fp64 accumulation in index order: identical to a plain Python loop
    for i in range(0, 64, 7):
        acc = 0.0
        for t in x[i]:
            acc += float(t)
        assert float(wide[i]) == acc


def test_sum_over_flipped_view_equals_sum_over_original():
    rng = rng_for(55)
    xi = random_view(rng, "int32", (40, 30))
    assert np.array_equal(_reduce("sum", xi, [0], "int64"), _reduce("sum", xi.flip(0), [0], "int64"))
    assert np.array_equal(_reduce("sum", xi, [1], "int64"), _reduce("sum", xi.flip(1).flip(0), [1], "int64")[::-1])
    # floats whose sums are exact (integers scaled by a power of two): order cannot matter
    xf = (rng.integers(-1000, 1000, size=(40, 30)) * 2.0 ** -7).astype(np.float32)
    v = View.from_numpy(xf)
    assert np.array_equal(_reduce("sum", v, [0], "float"), _reduce("sum", v.flip(0), [0], "float"))
    assert np.array_equal(_reduce("sum", v, [0, 1], "float"), _reduce("sum", v.flip(1).permute(1, 0), [0, 1], "float"))
    assert float(_reduce("sum", v, [0, 1], "float")) == float(xf.astype(np.float64).sum())


@pytest.mark.parametrize("dt", X.SIGNED + X.UNSIGNED + X.REAL + ("bool",))
@pytest.mark.parametrize("op", ("min", "max"))
def test_min_max_match_numpy_on_nan_free_data(dt, op):
    rng = rng_for(56)
    a = random_view(rng, dt, (7, 50, 3), specials=False).permute(2, 0, 1)
    arr = a.to_numpy()
    f = np.min if op == "min" else np.max
    for axes in ([2], [0], [0, 2], [0, 1, 2]):
        got = _reduce(op, a, axes, dt)
        assert np.array_equal(got, f(arr, axis=tuple(axes)))


def test_min_max_propagate_nan_and_order_signed_zeros():
    x = np.array([[1.0, math.nan, 3.0], [0.0, -0.0, -0.0], [-0.0, 0.0, -1.0], [-0.0, -0.0, -0.0]], dtype=np.float32)
    mx = _reduce("max", View.from_numpy(x), [1], "float")
    mn = _reduce("min", View.from_numpy(x), [1], "float")
    assert math.isnan(mx[0]) and math.isnan(mn[0])
    assert [math.copysign(1, float(t)) for t in mx[1:]] == [1.0, 1.0, -1.0] and mx[2] == 0.0
    assert mn[1] == 0.0 and math.copysign(1, float(mn[1])) == -1.0 and mn[2] == -1.0
    # result does not depend on the position of the NaN or the zero
    for perm in itertools.permutations(range(3)):
        y = x[:, list(perm)]
        assert np.array_equal(_reduce("max", View.from_numpy(y), [1], "float").view(np.uint32)[1:], mx.view(np.uint32)[1:])
        assert math.isnan(_reduce("min", View.from_numpy(y), [1], "float")[0])


def test_half_max_exact():
    rng = rng_for(57)
    x = rng.standard_normal((100, 333)).astype(np.float16)
    got = _reduce("max", View.from_numpy(x), [1], "half")
    assert np.array_equal(got.view(np.uint16), x.max(axis=1).view(np.uint16))


def test_prod_any_all():
    x = np.array([[1, 2, 3, 4], [5, 0, 7, 1], [-1, -1, -1, 2]], dtype=np.int16)
    assert list(_reduce("prod", View.from_numpy(x), [1], "int64")) == [24, 0, -2]
    assert list(_reduce("any", View.from_numpy(x), [0], "bool")) == [True, True, True, True]
    assert list(_reduce("all", View.from_numpy(x), [1], "bool")) == [True, False, True]
    f = np.array([[0.0, -0.0, math.nan], [0.0, 0.0, 0.0]], dtype=np.float64)
    assert list(_reduce("any", View.from_numpy(f), [1], "bool")) == [True, False]
    z = np.array([0j, 1j], dtype=np.complex64)
    assert bool(_reduce("any", View.from_numpy(z), [0], "bool")) is True
    assert bool(_reduce("all", View.from_numpy(z), [0], "bool")) is False
    p = np.array([1.5, 2.0, -4.0], dtype=np.float32)
    assert float(_reduce("prod", View.from_numpy(p), [0], "float")) == -12.0
    wrap = np.array([2 ** 62, 4], dtype=np.int64)
    assert int(_reduce("prod", View.from_numpy(wrap), [0], "int64")) == 0      # wraps modulo 2^64
    assert int(_reduce("sum", View.from_numpy(np.array([2 ** 63 - 1, 1], dtype=np.int64)), [0], "int64")) == -2 ** 63


def test_complex_sum_componentwise():
    rng = rng_for(58)
    z = random_view(rng, "cfloat", (20, 31), specials=False)
    got = _reduce("sum", z, [0], "cdouble")
    arr = z.to_numpy()
    for j in range(31):
        re = 0.0
        im = 0.0
        for i in range(20):
            re += float(arr[i, j].real)
            im += float(arr[i, j].imag)
        assert got[j] == complex(re, im)


def test_sum_result_conversion_saturates_like_a_cast():
    x = np.full(1000, 100, dtype=np.int8)
    assert int(_reduce("sum", View.from_numpy(x), [0], "int16")) == 32767
    assert int(_reduce("sum", View.from_numpy(x), [0], "int32")) == 100000
    assert float(_reduce("sum", View.from_numpy(x), [0], "float")) == 100000.0


def test_empty_and_degenerate():
    e = View.empty("float", (4, 0))
    assert list(_reduce("sum", e, [1], "float")) == [0.0, 0.0, 0.0, 0.0]
    assert list(_reduce("all", e, [1], "bool")) == [True] * 4
    assert list(_reduce("any", e, [1], "bool")) == [False] * 4
    assert list(_reduce("prod", e, [1], "float")) == [1.0] * 4
    with pytest.raises(O.OracleError) as err:
        _reduce("max", e, [1], "float")
    assert err.value.code == O.ERR_EMPTY
    assert _reduce("max", e, [0], "float").shape == (0,)            # no outputs: nothing to do
    # no axes: a cast copy
    rng = rng_for(59)
    v = random_view(rng, "float", (3, 4), specials=False)
    assert np.array_equal(_reduce("sum", v, [], "float"), v.to_numpy())
    # scalar (0-d) result of a full reduction
    assert _reduce("sum", v, [0, 1], "double").shape == ()
    with pytest.raises(O.OracleError):
        _reduce("sum", v, [0, 0], "double")
    with pytest.raises(O.OracleError):
        _reduce("sum", v, [2], "double")
