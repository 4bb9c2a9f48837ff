"""Pins for the oracle's elementary functions (sin, cos, tan, exp, log, the inverse and
hyperbolic functions, complex sqrt and the complex modulus): values
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
    if op in ("sinh", "cosh", "tanh"):
        s, c = d_sin_cos(y)
        ch, sh = (x.exp() + (-x).exp()) / 2, (x.exp() - (-x).exp()) / 2
        snh = (sh * c, ch * s)
        csh = (ch * c, sh * s)
        if op == "sinh":
            return snh
        if op == "cosh":
            return csh
        den = csh[0] ** 2 + csh[1] ** 2
        return ((snh[0] * csh[0] + snh[1] * csh[1]) / den, (snh[1] * csh[0] - snh[0] * csh[1]) / den)
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


@pytest.mark.parametrize("op", ("sinh", "cosh", "tanh"))
def test_complex_hyperbolic_functions_in_double(op):
    rng = rng_for(9004)
    z = rng.uniform(-6, 6, 120) + 1j * rng.uniform(-6, 6, 120)
    got = _oracle(op, z.astype(np.complex128), "cdouble")
    for zi, gi in zip(z, got):
        er, ei = d_complex(op, Decimal(float(zi.real)), Decimal(float(zi.imag)))
        mag = (er * er + ei * ei).sqrt()
        tol = mag * Decimal(2) ** -50
        assert abs(Decimal(float(gi.real)) - er) <= tol and abs(Decimal(float(gi.imag)) - ei) <= tol, (op, zi, gi)


FORWARD = {"asin": "sin", "acos": "cos", "atan": "tan"}


@pytest.mark.parametrize("op", ("asin", "acos", "atan"))
def test_complex_inverse_functions_invert_the_forward_function(op):
    # w = f^-1(z) is pinned through the forward function in arbitrary precision: f(w) must give z
    # back as closely as a few units in the last place of w allow (an error dw in w moves f(w) by
    # f'(w) dw), and w must lie in the principal range of the function.
    rng = rng_for(9005)
    z = np.concatenate([rng.uniform(-4, 4, 100) + 1j * rng.uniform(-4, 4, 100),
                        rng.uniform(-0.9, 0.9, 40) + 1j * rng.uniform(-0.3, 0.3, 40)])
    got = _oracle(op, z.astype(np.complex128), "cdouble")
    for zi, wi in zip(z, got):
        wr, wim = Decimal(float(wi.real)), Decimal(float(wi.imag))
        fr, fi = d_complex(FORWARD[op], wr, wim)
        # |f'(w)|: cos w for asin, sin w for acos, 1 + tan^2 w for atan
        if op == "asin":
            dr, di = d_complex("cos", wr, wim)
        elif op == "acos":
            dr, di = d_complex("sin", wr, wim)
        else:
            dr, di = 1 + fr * fr - fi * fi, 2 * fr * fi
        slope = (dr * dr + di * di).sqrt()
        wmag = (wr * wr + wim * wim).sqrt()
        tol = slope * wmag * Decimal(2) ** -50 + Decimal(10) ** -300
        err = ((fr - Decimal(float(zi.real))) ** 2 + (fi - Decimal(float(zi.imag))) ** 2).sqrt()
        assert err <= tol, (op, zi, wi, err, tol)
        if op == "acos":
            assert 0 <= wi.real <= np.pi
        else:
            assert -np.pi / 2 <= wi.real <= np.pi / 2
    if op in ("asin", "acos"):       # acos z + asin z = pi / 2
        other = _oracle("acos" if op == "asin" else "asin", z.astype(np.complex128), "cdouble")
        assert np.all(np.abs(got + other - np.pi / 2) <= 1e-15 * (1 + np.abs(got)))


def test_complex_inverse_and_hyperbolic_closed_forms_and_branch_cuts():
    def one(op, v):
        return _oracle(op, np.array([v], dtype=np.complex128), "cdouble")[0]
    assert one("asin", 0j) == 0 and one("acos", 0j).real == np.pi / 2 and one("atan", 1 + 0j).real == np.pi / 4
    w = one("asin", 1j)                                   # asin(i) = i asinh(1)
    assert w.real == 0 and abs(w.imag - 0.881373587019543) < 2e-16
    # the cuts of asin and acos run along the real axis beyond +-1; the sign of the zero
    # imaginary part selects the side (conjugate symmetry): asin(2 +- 0i) = pi/2 +- i ln(2 + sqrt 3)
    up, dn = one("asin", complex(2, 0.0)), one("asin", complex(2, -0.0))
    assert up.real == dn.real == np.pi / 2 and abs(up.imag - np.log(2 + np.sqrt(3))) < 4e-16 and dn.imag == -up.imag
    up, dn = one("acos", complex(2, 0.0)), one("acos", complex(2, -0.0))
    assert up.real == 0 and dn.real == 0 and up.imag == -dn.imag and up.imag < 0
    # atan: cuts along the imaginary axis beyond +-i; the sign of the zero real part selects the side
    rt, lf = one("atan", complex(0.0, 2)), one("atan", complex(-0.0, 2))
    assert rt.real == np.pi / 2 and lf.real == -np.pi / 2 and abs(rt.imag - np.arctanh(0.5)) < 2e-16 and lf.imag == rt.imag
    assert one("sinh", 0j) == 0 and one("cosh", 0j) == 1 and one("tanh", 0j) == 0
    w = one("sinh", 1j * np.pi / 2)
    assert abs(w.real) < 1e-16 and w.imag == 1.0
    w = one("cosh", 1j * np.pi)
    assert w.real == -1.0 and abs(w.imag) < 2e-16
    # sinh z = -i sin(iz), cosh z = cos(iz), tanh z = -i tan(iz), to the last bit (as C defines them)
    rng = rng_for(9006)
    z = (rng.uniform(-3, 3, 100) + 1j * rng.uniform(-3, 3, 100)).astype(np.complex128)
    assert np.array_equal(_oracle("sinh", z, "cdouble"), -1j * _oracle("sin", 1j * z, "cdouble"))
    assert np.array_equal(_oracle("cosh", z, "cdouble"), _oracle("cos", 1j * z, "cdouble"))


def test_complex_functions_of_infinite_and_nan_arguments_follow_the_c_standard():
    # the values C's Annex G prescribes for the exponential and the hyperbolic sine and cosine
    # (the trigonometric ones follow through sin z = -i sinh(iz), cos z = cosh(iz))
    inf, nan = np.inf, np.nan

    def one(op, re, im):
        return _oracle(op, np.array([complex(re, im)], dtype=np.complex128), "cdouble")[0]

    def same(w, re, im):
        def part(g, v):
            if v is None:
                return True
            if np.isnan(v):
                return bool(np.isnan(g))
            return g == v and np.signbit(g) == np.signbit(v)
        return part(w.real, re) and part(w.imag, im)
    assert same(one("exp", 0.0, 0.0), 1.0, 0.0) and same(one("exp", -0.0, -0.0), 1.0, -0.0)
    assert same(one("exp", 1.0, inf), nan, nan) and same(one("exp", 1.0, nan), nan, nan)
    assert same(one("exp", inf, 0.0), inf, 0.0) and same(one("exp", -inf, 1.0), 0.0 * np.cos(1.0), 0.0)
    assert same(one("exp", inf, 2.0), -inf, inf)                     # +inf cis(2): cos 2 < 0 < sin 2
    w = one("exp", -inf, inf)
    assert w.real == 0 and w.imag == 0                               # signs unspecified
    w = one("exp", inf, inf)
    assert np.isinf(w.real) and np.isnan(w.imag)
    assert same(one("exp", nan, 0.0), nan, 0.0) and same(one("exp", nan, 1.0), nan, nan)
    assert same(one("sinh", 0.0, inf), None, nan) and one("sinh", 0.0, inf).real == 0
    assert same(one("sinh", inf, 0.0), inf, 0.0) and same(one("sinh", inf, 2.0), -inf, inf)
    assert same(one("sinh", 1.0, inf), nan, nan) and same(one("sinh", nan, 0.0), nan, 0.0)
    assert same(one("cosh", 0.0, inf), nan, None) and one("cosh", 0.0, inf).imag == 0
    assert same(one("cosh", inf, 0.0), inf, 0.0) and same(one("cosh", inf, 2.0), -inf, inf)
    assert same(one("cosh", 1.0, inf), nan, nan)
    assert same(one("tanh", inf, 1.0), 1.0, 0.0) and same(one("tanh", inf, 2.0), 1.0, -0.0)   # 1 + i0 sin(2y)
    assert same(one("tanh", 0.0, inf), None, nan)
    assert same(one("cos", inf, 0.0), nan, None) and one("cos", inf, 0.0).imag == 0
    assert same(one("tan", 1.0, inf), 0.0, 1.0)                      # sin 2 > 0
    assert same(one("sin", 0.0, inf), 0.0, inf)


def test_complex_modulus():
    # |x + iy| = sqrt(x^2 + y^2), a real value of the input's precision, without undue overflow
    rng = rng_for(9007)
    z = (rng.uniform(-6, 6, 300) + 1j * rng.uniform(-6, 6, 300)) * np.exp(rng.uniform(-40, 40, 300))
    got = _oracle("abs", z.astype(np.complex128), "double")
    for zi, gi in zip(z, got):
        exact = (Decimal(float(zi.real)) ** 2 + Decimal(float(zi.imag)) ** 2).sqrt()
        assert abs(Decimal(float(gi)) - exact) <= Decimal(float(np.spacing(gi))), (zi, gi)
    def one(re, im, dt_in=np.complex128, dt_out="double"):
        return _oracle("abs", np.array([complex(re, im)], dtype=dt_in), dt_out)[0]
    assert one(3, 4) == 5 and one(-3, -4) == 5 and one(0.0, -0.0) == 0 and not np.signbit(one(-0.0, -0.0))
    assert one(1e200, 1e200) == np.hypot(1e200, 1e200) and np.isfinite(one(1e300, 1e300))
    assert one(3e-320, 4e-320) == 5e-320
    assert one(np.inf, np.nan) == np.inf and one(np.nan, -np.inf) == np.inf and np.isnan(one(np.nan, 1.0))
    # single-precision input: evaluated in single precision whatever the output type is
    zs = (rng.uniform(-6, 6, 200) + 1j * rng.uniform(-6, 6, 200)).astype(np.complex64)
    g32 = _oracle("abs", zs, "float")
    g64 = _oracle("abs", zs, "double")
    assert g32.dtype == np.float32 and np.array_equal(g32.astype(np.float64), g64)
    exact = np.hypot(zs.real.astype(np.float64), zs.imag.astype(np.float64))
    assert np.all(np.abs(g32.astype(np.float64) - exact) <= np.spacing(g32).astype(np.float64) * 0.5000001)
    # complex output: the modulus with a zero imaginary part
    gc = _oracle("abs", zs, "cfloat")
    assert np.array_equal(gc.real, g32) and np.all(gc.imag == 0)
    # strict types accept the real type of the same precision only
    a = View.from_numpy(zs)
    O.unary("abs", a, View.empty("float", zs.shape), O.STRICT_TYPES)
    with pytest.raises(O.OracleError):
        O.unary("abs", a, View.empty("double", zs.shape), O.STRICT_TYPES)


def test_not_defined_for_integers():
    with pytest.raises(O.OracleError):
        O.unary("sin", View.empty("int32", (3,)), View.empty("int32", (3,)))
