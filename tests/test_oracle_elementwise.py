"""Pins for the oracle's elementwise unary and binary operations.

Three independent references: (1) the exact-rational per-index brute force of tests/brute.py
on tiny strided tensors for every operation and compute type; (2) numpy on materialised
copies for the cases where numpy's routine has the same definition (IEEE add/sub/mul/div in
float32/float64, wrapping integer arithmetic, comparisons); (3) hand-computed values.
"""
import itertools
import math

import numpy as np
import pytest

import brute
import exactmath as X
from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import DTYPES, View


def _strided_pair(rng, da, db, dout, sizes=(3, 4, 5)):
    """a: permuted + stepped; b: broadcast along one axis and reversed; out: column-major."""
    s0, s1, s2 = sizes
    a = random_view(rng, da, (s2, s0, 2 * s1)).permute(1, 2, 0).slice(1, 0, 2 * s1, 2)
    b = random_view(rng, db, (s0, 1, s2)).flip(2)
    out = View.empty(dout, sizes, order="F")
    return a, b, out


def _cases_binary():
    cases = []
    for T in X.ALL:
        for op in X.ARITH + X.BITWISE:
            if X.binary_supported(op, T):
                cases.append((op, T, T, T))
    # mixed inputs converted to the output type
    for op in ("add", "mul", "sub", "div", "max"):
        cases += [(op, "int32", "float", "float"), (op, "double", "int8", "int16"),
                  (op, "half", "uint8", "half"), (op, "int64", "double", "float"),
                  (op, "cfloat", "half", "chalf"), (op, "bool", "int16", "double")]
    # destinations that are neither an operand's type nor able to hold the promoted type: the
    # operation runs in the promoted type and its result is converted once
    for op in ("add", "sub", "mul", "div", "min"):
        cases += [(op, "int32", "int32", "int8"), (op, "double", "double", "float"),
                  (op, "int16", "uint8", "int8"), (op, "float", "int32", "half"),
                  (op, "uint64", "int8", "uint16"), (op, "cdouble", "float", "cfloat"),
                  (op, "half", "half", "int16"), (op, "chalf", "half", "half"), (op, "half", "uint8", "int32")]
    for op in X.BITWISE:
        cases += [(op, "int32", "uint8", "int8"), (op, "uint16", "bool", "uint8")]
    cases = [c for c in cases if X.binary_supported(c[0], X.compute_type(*c))]
    for op in X.COMPARE + X.LOGICAL:
        for da, db in [("int8", "uint8"), ("int64", "uint64"), ("int64", "float"), ("half", "int16"),
                       ("float", "double"), ("bool", "half"), ("cfloat", "cdouble"), ("chalf", "int32"),
                       ("uint32", "int32"), ("double", "double"), ("int16", "int16"), ("chalf", "chalf"),
                       ("cdouble", "cdouble"), ("uint64", "uint64"), ("half", "half")]:
            T = X.compute_type(op, da, db, "bool")
            if X.binary_supported(op, T):
                cases.append((op, da, db, "bool"))
        cases.append((op, "float", "float", "int32"))  # non-bool destination of a predicate
    return cases


@pytest.mark.parametrize("op,da,db,dout", _cases_binary())
def test_binary_against_exact_rational_brute_force(op, da, db, dout):
    rng = rng_for(4000 + sum(map(ord, op + da + db + dout)))
    a, b, out = _strided_pair(rng, da, db, dout)
    want = brute.binary(op, a, b, out)
    O.binary(op, a, b, out)
    assert brute.storages_match(dout, out.storage, want, out)


@pytest.mark.parametrize("op,T", [(op, T) for op in X.UNARY for T in X.ALL if X.unary_supported(op, "bool" if op == "lnot" else T)])
def test_unary_against_exact_rational_brute_force(op, T):
    rng = rng_for(5000 + sum(map(ord, op + T)))
    a = random_view(rng, T, (4, 3, 5)).permute(2, 1, 0).flip(0)
    out = View.empty(T, a.sizes, order="F")
    want = brute.unary(op, a, out)
    O.unary(op, a, out)
    assert brute.storages_match(T, out.storage, want, out)


@pytest.mark.parametrize("dt", ("float", "double"))
@pytest.mark.parametrize("op", ("add", "sub", "mul", "div"))
def test_ieee_arithmetic_matches_numpy(dt, op):
    rng = rng_for(41)
    a = random_view(rng, dt, (50, 40))
    b = random_view(rng, dt, (40, 50)).permute(1, 0)
    out = View.empty(dt, (50, 40))
    O.binary(op, a, b, out)
    f = {"add": np.add, "sub": np.subtract, "mul": np.multiply, "div": np.divide}[op]
    with np.errstate(all="ignore"):
        want = f(a.to_numpy(), b.to_numpy())
    got = out.to_numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    u = np.uint32 if dt == "float" else np.uint64
    assert np.array_equal(got[~nan].view(u), want[~nan].view(u))


@pytest.mark.parametrize("dt", X.SIGNED + X.UNSIGNED)
@pytest.mark.parametrize("op", ("add", "sub", "mul"))
def test_integer_arithmetic_wraps_like_numpy(dt, op):
    rng = rng_for(42)
    a = random_view(rng, dt, (30, 20))
    b = random_view(rng, dt, (30, 20)).flip(0)
    out = View.empty(dt, (30, 20))
    O.binary(op, a, b, out)
    f = {"add": np.add, "sub": np.subtract, "mul": np.multiply}[op]
    with np.errstate(over="ignore"):
        assert np.array_equal(out.to_numpy(), f(a.to_numpy(), b.to_numpy()))


@pytest.mark.parametrize("dt", ("int32", "uint16", "float", "double", "half"))
@pytest.mark.parametrize("op", ("eq", "ne", "lt", "le", "gt", "ge"))
def test_comparisons_match_numpy(dt, op):
    rng = rng_for(43)
    a = random_view(rng, dt, (500,))
    b = random_view(rng, dt, (500,))
    b.storage[:400] = a.storage[:400]  # plenty of equal pairs
    out = View.empty("bool", (500,))
    O.binary(op, a, b, out)
    f = {"eq": np.equal, "ne": np.not_equal, "lt": np.less, "le": np.less_equal,
         "gt": np.greater, "ge": np.greater_equal}[op]
    assert np.array_equal(out.to_numpy(), f(a.to_numpy(), b.to_numpy()))


def test_complex_multiply_hand_values():
    # (1+2i)(3+4i) = -5+10i ; i*i = -1 ; real*real stays real ; conj symmetry
    a = np.array([1 + 2j, 1j, 3 + 0j, 2 - 3j], dtype=np.complex64)
    b = np.array([3 + 4j, 1j, -2 + 0j, 5 + 7j], dtype=np.complex64)
    out = View.empty("cfloat", (4,))
    O.binary("mul", View.from_numpy(a), View.from_numpy(b), out)
    got = out.to_numpy()
    assert list(got[:3]) == [-5 + 10j, -1 + 0j, -6 + 0j]
    assert got[3] == (2 * 5 + 3 * 7) + (2 * 7 - 3 * 5) * 1j
    out2 = View.empty("cfloat", (4,))
    O.binary("mul", View.from_numpy(np.conj(a)), View.from_numpy(np.conj(b)), out2)
    assert np.array_equal(out2.to_numpy(), np.conj(got))


def test_complex_multiply_rounds_each_of_six_operations():
    # products that are inexact in float32: a fused multiply-add would change the last bit
    a = np.array([1.0000001 + 3.3333333j], dtype=np.complex64)
    b = np.array([7.7777777 + 1.2345678j], dtype=np.complex64)
    out = View.empty("cfloat", (1,))
    O.binary("mul", View.from_numpy(a), View.from_numpy(b), out)
    f = np.float32
    ar, ai, br, bi = f(a.real[0]), f(a.imag[0]), f(b.real[0]), f(b.imag[0])
    re = f(f(ar * br) - f(ai * bi))
    im = f(f(ar * bi) + f(ai * br))
    g = out.to_numpy()[0]
    assert f(g.real) == re and f(g.imag) == im
    # and it does differ from the exactly-computed-then-rounded product in at least one case
    rng = rng_for(44)
    a = random_view(rng, "cfloat", (2000,), specials=False)
    b = random_view(rng, "cfloat", (2000,), specials=False)
    out = View.empty("cfloat", (2000,))
    O.binary("mul", a, b, out)
    exact = (a.to_numpy().astype(np.complex128) * b.to_numpy().astype(np.complex128)).astype(np.complex64)
    assert (out.to_numpy() != exact).any()


def test_absgt_complex_uses_squared_magnitudes_in_double():
    a = np.array([3 + 4j, 1 + 1j, 0j, complex(math.nan, 0), 5 + 0j], dtype=np.complex64)
    b = np.array([4 + 3j, 1 - 1j, 1e-30 + 0j, 1 + 0j, complex(3, math.nan)], dtype=np.complex64)
    out = View.empty("bool", (5,))
    O.binary("absgt", View.from_numpy(a), View.from_numpy(b), out)
    assert list(out.to_numpy()) == [False, False, False, False, False]
    O.binary("absgt", View.from_numpy(b), View.from_numpy(a), out)
    assert list(out.to_numpy()) == [False, False, True, False, False]
    # a defined tie: magnitudes that differ by less than one unit in the last place of the
    # double-precision sum compare as equal (documented behaviour of the squared-magnitude rule)
    big = np.float32(4096.0)
    tiny = np.float32(2.0 ** -20)
    a = np.array([complex(big, tiny)], dtype=np.complex64)   # |a|^2 = 2^24 + 2^-40 -> rounds to 2^24
    b = np.array([complex(big, 0.0)], dtype=np.complex64)
    o1 = View.empty("bool", (1,))
    O.binary("absgt", View.from_numpy(a), View.from_numpy(b), o1)
    assert list(o1.to_numpy()) == [False]


def test_absgt_signed_minimum():
    a = np.array([-128, 127, -5], dtype=np.int8)
    b = np.array([127, -128, 5], dtype=np.int8)
    out = View.empty("bool", (3,))
    O.binary("absgt", View.from_numpy(a), View.from_numpy(b), out)
    assert list(out.to_numpy()) == [True, False, False]


def test_min_max_nan_and_signed_zero():
    a = np.array([math.nan, 1.0, 0.0, -0.0, -0.0, 2.0], dtype=np.float32)
    b = np.array([1.0, math.nan, -0.0, 0.0, -0.0, 3.0], dtype=np.float32)
    out = View.empty("float", (6,))
    O.binary("max", View.from_numpy(a), View.from_numpy(b), out)
    g = out.to_numpy()
    assert math.isnan(g[0]) and math.isnan(g[1])
    assert [math.copysign(1, float(t)) for t in g[2:5]] == [1.0, 1.0, -1.0] and g[5] == 3.0
    O.binary("min", View.from_numpy(a), View.from_numpy(b), out)
    g = out.to_numpy()
    assert math.isnan(g[0]) and math.isnan(g[1])
    assert [math.copysign(1, float(t)) for t in g[2:5]] == [-1.0, -1.0, -1.0] and g[5] == 2.0


def test_integer_division_rules():
    a = np.array([7, -7, 7, -7, -128, 5, 0, 5, -9, 127], dtype=np.int8)
    b = np.array([2, 2, -2, -2, -1, 0, 0, -1, -1, -1], dtype=np.int8)
    out = View.empty("int8", (10,))
    O.binary("div", View.from_numpy(a), View.from_numpy(b), out)
    assert list(out.to_numpy()) == [3, -3, -3, 3, -128, 0, 0, -5, 9, -127]
    for dt in ("int16", "int32", "int64"):
        lo = -2 ** (8 * np.dtype(dt).itemsize - 1)
        a = np.array([lo, lo + 1, 11, lo], dtype=dt)
        b = np.array([-1, -1, -1, 2], dtype=dt)
        out = View.empty(dt, (4,))
        O.binary("div", View.from_numpy(a), View.from_numpy(b), out)
        assert [int(t) for t in out.to_numpy()] == [lo, -(lo + 1), -11, lo // 2]


def test_operand_types_set_the_compute_type_when_the_destination_is_narrower():
    """Section 3.2.1: the operation's type is the smallest one holding both operands' types.  A
    destination of another, narrower type receives that result converted once; it does not
    narrow the operands first.  Values worked by hand."""
    i32 = lambda *v: View.from_numpy(np.array(v, dtype=np.int32))
    out = View.empty("int8", (3,))
    O.binary("add", i32(1000, -1000, 100), i32(-900, 900, 100), out)
    assert list(out.to_numpy()) == [100, -100, 127]          # sat(1000) + sat(-900) would be -1
    O.binary("bxor", i32(0x1FF, 0x7FFFFFFF, 3), i32(0x180, 0x7FFFFF00, 1), out)
    assert list(out.to_numpy()) == [0x7F, 127, 2]            # 127 ^ 127 would be 0
    O.binary("mul", i32(100, 16, -16), i32(100, 8, 8), out)
    assert list(out.to_numpy()) == [127, 127, -128]
    # one rounding: (1 + 2^-24 + 2^-30) + (-2^-30) = 1 + 2^-24 exactly, a tie that rounds to 1;
    # narrowing the first operand to single precision before adding would give 1 + 2^-23
    a = View.from_numpy(np.array([1 + 2.0 ** -24 + 2.0 ** -30], dtype=np.float64))
    b = View.from_numpy(np.array([-(2.0 ** -30)], dtype=np.float64))
    o = View.empty("float", (1,))
    O.binary("add", a, b, o)
    assert o.to_numpy()[0] == np.float32(1.0)
    assert np.float32(a.to_numpy()[0]) + np.float32(b.to_numpy()[0]) == np.float32(1 + 2.0 ** -23)
    # the destination's type still rules when it is an operand's type (A += B) ...
    acc = View.from_numpy(np.array([100, -100], dtype=np.int8))
    O.binary("add", acc, i32(1000, -1000), acc)
    assert list(acc.to_numpy()) == [-29, 28]                 # 100 + sat(1000) = 227 wraps; -100 - 128 wraps
    # ... and when it holds the promoted type (int8 and uint8 promote to int16, held by int64)
    wide = View.empty("int64", (1,))
    O.binary("mul", View.from_numpy(np.array([-128], dtype=np.int8)),
             View.from_numpy(np.array([255], dtype=np.uint8)), wide)
    assert int(wide.to_numpy()[0]) == -32640


def test_config3_both_compute_type_readings_agree():
    """int32 (|a| <= 1000) times float32: computing in float32 (destination type) and computing
    in the promoted type double then rounding once give identical bits, because a*b is exact in
    double."""
    rng = rng_for(45)
    a = rng.integers(-1000, 1000, size=(64, 257), endpoint=True).astype(np.int32)
    b = rng.standard_normal((1, 257)).astype(np.float32)
    va, vb = View.from_numpy(a), View.from_numpy(b)
    assert O.promote("int32", "float") == "double"
    out32 = View.empty("float", (64, 257))
    O.binary("mul", va, vb, out32)
    out64 = View.empty("double", (64, 257))
    O.binary("mul", va, vb, out64)
    narrowed = View.empty("float", (64, 257))
    O.cast_copy(out64, narrowed)
    assert np.array_equal(out32.storage, narrowed.storage)
    assert np.array_equal(out32.to_numpy(), a.astype(np.float32) * b)


def test_unsupported_combinations_are_rejected():
    f = View.from_numpy(np.zeros(3, dtype=np.float32))
    c = View.from_numpy(np.zeros(3, dtype=np.complex64))
    b = View.from_numpy(np.zeros(3, dtype=np.bool_))
    for op, x, y, o in [("band", f, f, f), ("lt", c, c, b), ("max", c, c, c), ("add", b, b, b)]:
        with pytest.raises(O.OracleError) as e:
            O.binary(op, x, y, o.fresh_copy())
        assert e.value.code == O.ERR_DTYPE
    with pytest.raises(O.OracleError):
        O.unary("abs", b, b.fresh_copy())       # no modulus in bool arithmetic
    with pytest.raises(O.OracleError):
        O.unary("bnot", c, c.fresh_copy())
    i = View.from_numpy(np.zeros(3, dtype=np.int32))
    with pytest.raises(O.OracleError):
        O.unary("sqrt", i, i.fresh_copy())


def test_strict_types_flag():
    a = View.from_numpy(np.zeros(3, dtype=np.int32))
    b = View.from_numpy(np.zeros(3, dtype=np.float32))
    out = View.empty("float", (3,))
    with pytest.raises(O.OracleError) as e:
        O.binary("add", a, b, out, flags=O.STRICT_TYPES)
    assert e.value.code == O.ERR_DTYPE
    O.binary("add", b, b, out, flags=O.STRICT_TYPES)


def test_shape_errors():
    a = View.from_numpy(np.zeros((2, 3), dtype=np.float32))
    b = View.from_numpy(np.zeros((3, 2), dtype=np.float32))
    with pytest.raises(O.OracleError) as e:
        O.binary("add", a, b, View.empty("float", (2, 3)))
    assert e.value.code == O.ERR_SHAPE


def test_byte_swap_matches_numpy_and_is_an_involution():
    rng = rng_for(77)
    for dt, npdt in (("int16", np.int16), ("uint16", np.uint16), ("int32", np.int32), ("uint32", np.uint32),
                     ("int64", np.int64), ("uint64", np.uint64), ("int8", np.int8), ("uint8", np.uint8)):
        x = rng.integers(np.iinfo(npdt).min, np.iinfo(npdt).max, size=(7, 9), dtype=npdt, endpoint=True)
        a = View.from_numpy(x).permute(1, 0)
        out = View.empty(dt, a.sizes)
        O.unary("bswap", a, out)
        assert np.array_equal(out.to_numpy(), a.to_numpy().byteswap())
        back = View.empty(dt, a.sizes)
        O.unary("bswap", out, back)
        assert np.array_equal(back.to_numpy(), a.to_numpy())
    # a float stored in the other byte order, viewed as unsigned integers of its size
    f = np.array([1.5, -2.25, 3e10], dtype=np.float32)
    swapped = View.from_numpy(f.byteswap().view(np.uint32))
    out = View.empty("uint32", (3,))
    O.unary("bswap", swapped, out)
    assert np.array_equal(out.to_numpy().view(np.float32), f)
    with pytest.raises(O.OracleError):
        O.unary("bswap", View.from_numpy(f), View.empty("float", (3,)))


def test_domain_check():
    rng = rng_for(78)
    x = np.abs(rng.standard_normal((40, 30))).astype(np.float32)
    assert not O.domain_check("sqrt", View.from_numpy(x))
    assert not O.domain_check("log", View.from_numpy(x).permute(1, 0))
    x[17, 3] = -1e-30
    assert O.domain_check("sqrt", View.from_numpy(x)) and O.domain_check("log", View.from_numpy(x))
    assert not O.domain_check("exp", View.from_numpy(x))
    y = np.array([0.0, -0.0, np.nan, np.inf], dtype=np.float64)       # zeros, NaN and +Inf are inside the domain
    assert not O.domain_check("sqrt", View.from_numpy(y))
    assert O.domain_check("sqrt", View.from_numpy(np.array([-np.inf])))
    assert O.domain_check("log", View.from_numpy(np.array([3, -1, 2], dtype=np.int32)))
    # the inverse sine and cosine are defined on [-1, 1]
    u = rng.uniform(-1, 1, (30, 20)).astype(np.float32)
    u[0, 0], u[29, 19] = 1.0, -1.0
    assert not O.domain_check("acos", View.from_numpy(u)) and not O.domain_check("asin", View.from_numpy(u))
    u[11, 7] = np.float32(-1.0000001)
    assert O.domain_check("acos", View.from_numpy(u)) and O.domain_check("asin", View.from_numpy(u).permute(1, 0))
    assert not O.domain_check("atan", View.from_numpy(u)) and not O.domain_check("tanh", View.from_numpy(u))
    assert O.domain_check("asin", View.from_numpy(np.array([0, 2, 1], dtype=np.int16)))
    assert not O.domain_check("asin", View.from_numpy(np.array([np.nan, 0.5], dtype=np.float64)))
