"""Pins for the oracle's elementary functions (sin, cos, tan, exp, log, complex sqrt): values
computed independently of the C library with Python's arbitrary-precision `decimal` arithmetic
(Taylor series after argument reduction; exp and ln are decimal's own), closed forms and
identities.  The oracle must sit within one unit in the last place of the true value in double
precision (a few for the complex routines), and be the correct rounding to single in all but
rare double-rounding cases."""
from decimal import Decimal, getcontext

import numpy as np
import pytest

from oracle import binding as O
from workloads.values import rng_for
from workloads.views import View

getcontext().prec = 70
PI = Decimal("3.14159265358979323846264338327950288419716939937510582097494459230781640628620899")


def d_sin_cos(x: Decimal):
    k = (x / (2 * PI)).to_integral_value()
    r = x - k * 2 * PI
    # Taylor series of sin and cos at r (|r| <= pi)
    s, c = Decimal(0), Decimal(0)
    term = Decimal(1)
    n = 0
    while abs(term) > Decimal(10) ** -65:
        if n % 2 == 0:
            c += term if (n // 2) % 2 == 0 else -term
        else:
            s += term if (n // 2) % 2 == 0 else -term
        n += 1
        term = term * r / n
    return s, c


def d_atan(t: Decimal) -> Decimal:
    halvings = 0
    while abs(t) > Decimal("0.1"):
        t = t / (1 + (1 + t * t).sqrt())
        halvings += 1
    s, term, n, t2 = Decimal(0), t, 1, t * t
    while abs(term) > Decimal(10) ** -66:
        s += term / n if (n // 2) % 2 == 0 else -term / n
        term *= t2
        n += 2
    return s * (2 ** halvings)


def d_atan2(y: Decimal, x: Decimal) -> Decimal:
    if x > 0:
        return d_atan(y / x)
    if x < 0:
        return d_atan(y / x) + (PI if y >= 0 else -PI)
    return PI / 2 if y > 0 else -PI / 2


def d_real(op: str, x: Decimal) -> Decimal:
    if op == "sin":
        return d_sin_cos(x)[0]
    if op == "cos":
        return d_sin_cos(x)[1]
    if op == "tan":
        s, c = d_sin_cos(x)
        return s / c
    if op == "exp":
        return x.exp()
    if op == "log":
        return x.ln()
    if op == "atan":
        return d_atan(x)
    if op in ("asin", "acos"):
        if abs(x) == 1:
            a = PI / 2 if x > 0 else -PI / 2
        else:
            a = d_atan(x / (1 - x * x).sqrt())
        return a if op == "asin" else PI / 2 - a
    e, f = x.exp(), (-x).exp()
    if op == "sinh":
        return (e - f) / 2
    if op == "cosh":
        return (e + f) / 2
    return (e - f) / (e + f)


def d_complex(op: str, x: Decimal, y: Decimal):
    if op in ("sin", "cos", "tan"):
        s, c = d_sin_cos(x)
        ch, sh = (y.exp() + (-y).exp()) / 2, (y.exp() - (-y).exp()) / 2
        sn = (s * ch, c * sh)
        cs = (c * ch, -s * sh)
        if op == "sin":
            return sn
        if op == "cos":
            return cs
        den = cs[0] ** 2 + cs[1] ** 2
        return ((sn[0] * cs[0] + sn[1] * cs[1]) / den, (sn[1] * cs[0] - sn[0] * cs[1]) / den)
    if op == "exp":
        s, c = d_sin_cos(y)
        return (x.exp() * c, x.exp() * s)
    if op == "log":
        return ((x * x + y * y).ln() / 2, d_atan2(y, x))
    m = (x * x + y * y).sqrt()       # sqrt, principal branch
    t = ((abs(x) + m) / 2).sqrt()
    if x >= 0:
        return (t, y / (2 * t))
    return (abs(y) / (2 * t), t if y >= 0 else -t)


def _oracle(op, arr, dtype):
    a = View.from_numpy(arr)
    out = View.empty(dtype, arr.shape)
    O.unary(op, a, out)
    return out.to_numpy()


def _inputs(rng, op, n):
    if op in ("asin", "acos"):
        return rng.uniform(-1, 1, n)
    if op in ("sinh", "cosh", "tanh"):
        return rng.uniform(-12, 12, n)
    if op == "log":
        return np.exp(rng.uniform(-30, 30, n))
    if op == "exp":
        return rng.uniform(-60, 60, n)
    return rng.uniform(-40, 40, n)


REAL_OPS = ("sin", "cos", "tan", "exp", "log", "asin", "acos", "atan", "sinh", "cosh", "tanh")


@pytest.mark.parametrize("op", REAL_OPS)
def test_real_functions_in_double_within_one_ulp_of_the_true_value(op):
    x = _inputs(rng_for(9000), op, 150)
    got = _oracle(op, x, "double")
    for xi, gi in zip(x, got):
        exact = d_real(op, Decimal(float(xi)))
        ulp = Decimal(float(np.spacing(abs(gi))))
        # the C library documents up to two units in the last place for the hyperbolic functions
        assert abs(Decimal(float(gi)) - exact) <= (2 if op in ("sinh", "cosh", "tanh") else 1) * ulp, (op, xi, gi)


@pytest.mark.parametrize("op", REAL_OPS)
def test_real_functions_in_single_are_the_rounded_true_value(op):
    x = _inputs(rng_for(9001), op, 300).astype(np.float32)
    if op == "exp":
        x = np.clip(x, -80, 80)
    got = _oracle(op, x, "float")
    same = 0
    for xi, gi in zip(x, got):
        exact = d_real(op, Decimal(float(xi)))
        rn = np.float32(float(exact))          # float(Decimal) rounds correctly to double, then to single
        ulp = float(np.spacing(np.abs(rn)))
        assert abs(float(gi) - float(rn)) <= ulp, (op, xi, gi, rn)
        same += float(gi) == float(rn)
    assert same >= 297                          # double rounding may differ in rare cases only


def test_half_goes_through_single():
    x = np.linspace(-6, 6, 200).astype(np.float16)
    got = _oracle("sin", x, "half")
    want = np.sin(x.astype(np.float64)).astype(np.float32).astype(np.float16)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("op", ("sin", "cos", "tan", "exp", "log", "sqrt"))
def test_complex_functions_in_double(op):
    rng = rng_for(9002)
    z = rng.uniform(-6, 6, 120) + 1j * rng.uniform(-6, 6, 120)
    got = _oracle(op, z.astype(np.complex128), "cdouble")
    for zi, gi in zip(z, got):
        er, ei = d_complex(op, Decimal(float(zi.real)), Decimal(float(zi.imag)))
        mag = (er * er + ei * ei).sqrt()
        tol = mag * Decimal(2) ** -50                      # four units in the last place of |w|
        assert abs(Decimal(float(gi.real)) - er) <= tol and abs(Decimal(float(gi.imag)) - ei) <= tol, (op, zi, gi)


def test_closed_forms_and_branches():
    def one(op, v, dtype):
        return _oracle(op, np.array([v], dtype={"double": np.float64, "cdouble": np.complex128}[dtype]), dtype)[0]
    assert one("sin", 0.0, "double") == 0.0 and one("cos", 0.0, "double") == 1.0
    assert one("exp", 0.0, "double") == 1.0 and one("log", 1.0, "double") == 0.0
    assert one("exp", 1.0, "double") == 2.718281828459045
    assert np.isnan(one("log", -1.0, "double")) and one("log", 0.0, "double") == -np.inf
    assert np.isnan(one("sin", np.inf, "double"))
    assert one("asin", 1.0, "double") == np.pi / 2 and one("acos", -1.0, "double") == np.pi
    assert np.isnan(one("acos", 1.5, "double")) and np.isnan(one("asin", -1.0000001, "double"))
    assert one("atan", np.inf, "double") == np.pi / 2 and one("tanh", -np.inf, "double") == -1.0
    assert one("cosh", 0.0, "double") == 1.0 and one("sinh", -0.0, "double") == 0.0
    assert one("sqrt", complex(-1, 0.0), "cdouble") == 1j and one("sqrt", complex(-1, -0.0), "cdouble") == -1j   # branch cut
    assert one("sqrt", -4 + 0j, "cdouble") == 2j
    w = one("log", -1 + 0j, "cdouble")
    assert w.real == 0.0 and w.imag == np.pi
    w = one("exp", 1j * np.pi, "cdouble")
    assert w.real == -1.0 and abs(w.imag) < 2e-16


def test_identities():
    rng = rng_for(9003)
    x = rng.uniform(-20, 20, 500)
    s, c = _oracle("sin", x, "double"), _oracle("cos", x, "double")
    assert np.all(np.abs(s * s + c * c - 1) <= 4e-16)
    e = _oracle("exp", x, "double")
    assert np.all(np.abs(_oracle("log", e, "double") - x) <= 1e-15 * np.maximum(1, np.abs(x)))
    z = (rng.uniform(-3, 3, 200) + 1j * rng.uniform(-3, 3, 200)).astype(np.complex128)
    r = _oracle("sqrt", z, "cdouble")
    assert np.all(np.abs(r * r - z) <= 1e-15 * np.abs(z)) and np.all(r.real >= 0)


def test_inverse_and_hyperbolic_functions_are_real_only():
    z = View.from_numpy(np.zeros(3, dtype=np.complex64))
    for op in ("asin", "acos", "atan", "sinh", "cosh", "tanh"):
        with pytest.raises(O.OracleError):
            O.unary(op, z, z.fresh_copy())


def test_not_defined_for_integers():
    with pytest.raises(O.OracleError):
        O.unary("sin", View.empty("int32", (3,)), View.empty("int32", (3,)))
