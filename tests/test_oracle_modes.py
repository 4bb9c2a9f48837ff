"""Pins for the compute modes of section 3.2.1 of the paper (standard, warning, error, complex)
as the oracle composes them: the paper's own examples - the square root of negative reals and
the arccosine of magnitudes above one - with results known in closed form."""
import numpy as np
import pytest

from oracle import binding as O
from workloads.views import View


def _views(x, cdt="cdouble"):
    a = View.from_numpy(np.asarray(x, dtype=np.float64))
    return a, View.empty("double", a.sizes), View.empty(cdt, a.sizes)


def test_square_root_of_negative_reals():
    a, out, outc = _views([4.0, -4.0, 0.0, -0.0, np.nan])
    r = O.unary_mode("sqrt", "standard", a, out)
    assert r == {"outside": None, "wrote": "out"}
    got = out.to_numpy()
    assert got[0] == 2 and np.isnan(got[1]) and got[2] == 0 and np.isnan(got[4])
    r = O.unary_mode("sqrt", "warning", a, out.fresh_copy())
    assert r == {"outside": True, "wrote": "out"}
    untouched = out.fresh_copy()
    untouched.storage[:] = 0x77
    with pytest.raises(O.DomainError):
        O.unary_mode("sqrt", "error", a, untouched)
    assert np.all(untouched.storage == 0x77)                  # nothing was computed
    r = O.unary_mode("sqrt", "complex", a, out, outc)
    assert r == {"outside": True, "wrote": "out_complex"}
    z = outc.to_numpy()
    assert z[0] == 2 and z[1] == 2j and z[2] == 0 and np.isnan(z[4].real)
    # inside the domain every mode gives the real result (zeros, NaN and +Inf are inside)
    a, out, outc = _views([4.0, 0.0, -0.0, np.inf, np.nan, 2.25])
    for mode in O.MODES:
        o = out.fresh_copy()
        r = O.unary_mode("sqrt", mode, a, o, outc)
        assert r["wrote"] == "out" and r["outside"] in (None, False)
        got = o.to_numpy()
        assert got[0] == 2 and got[5] == 1.5 and np.isinf(got[3]) and np.isnan(got[4])


def test_arccosine_of_magnitudes_above_one():
    a, out, outc = _views([0.5, 2.0, -2.0, 1.0])
    O.unary_mode("acos", "standard", a, out)
    got = out.to_numpy()
    assert abs(got[0] - np.pi / 3) < 1e-15 and np.isnan(got[1]) and np.isnan(got[2]) and got[3] == 0
    assert O.unary_mode("acos", "warning", a, out.fresh_copy())["outside"] is True
    with pytest.raises(O.DomainError):
        O.unary_mode("acos", "error", a, out.fresh_copy())
    r = O.unary_mode("acos", "complex", a, out, outc)
    assert r["wrote"] == "out_complex"
    z = outc.to_numpy()
    # acos(2) = -i acosh(2) on the side of the cut a +0 imaginary part selects; acos(-2) = pi - i acosh(2)
    assert abs(z[0] - np.pi / 3) < 1e-15 and z[1].real == 0 and abs(z[1].imag + np.arccosh(2)) < 4e-16
    assert abs(z[2].real - np.pi) < 1e-15 and abs(z[2].imag + np.arccosh(2)) < 4e-16
    # magnitude exactly one is inside the domain
    a, out, outc = _views([1.0, -1.0, 0.25])
    assert O.unary_mode("acos", "error", a, out)["outside"] is False
    # operations defined everywhere are never outside
    a, out, outc = _views([-3.0, 3.0])
    assert O.unary_mode("sin", "error", a, out)["outside"] is False
    assert O.unary_mode("log", "complex", a, out, outc)["wrote"] == "out_complex"
    z = outc.to_numpy()
    assert abs(z[0] - complex(np.log(3), np.pi)) < 1e-15      # log(-3 + 0i) = log 3 + i pi
