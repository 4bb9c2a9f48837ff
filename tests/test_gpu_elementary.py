"""GPU parity of the elementary functions (sin, cos, tan, exp, log, complex sqrt) against the
oracle, in the tolerance class these operations have: a few units in the last place of the
output type (real: |gpu - oracle| <= K ulp of the oracle value; complex: each component within
K ulp of the magnitude of the oracle value).  Results of finite arguments agree with the
oracle in kind (NaN, signed infinity, signed zero), and so does the complex square root for
infinite parts.  Not compared: sin, cos, tan and exp of complex arguments with an infinite or
NaN part, where the kernels evaluate the plain formulas (e.g. exp(Inf + i Inf) gives NaN + i NaN,
C gives Inf + i NaN; cos(Inf + i0) gives NaN - i0, C gives NaN + i0; tan(Inf + i Inf) gives
NaN + i, C gives 0 + i)."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu

REAL = {"half": np.float16, "float": np.float32, "double": np.float64}
CPLX = {"chalf": np.float16, "cfloat": np.float32, "cdouble": np.float64}
K_ULP = {"half": 1, "float": 4, "double": 4, "chalf": 2, "cfloat": 8, "cdouble": 8}


def _run(op, a: View, out: View):
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = H.DeviceViews()
    ta, to = dv.tensor(a), dv.tensor(out)
    ocn.unary(op, ta, to)
    dv.torch.cuda.synchronize()
    got_storage = dv.download(out).copy()
    O.unary(op, a, out)
    got = View(got_storage, out.dtype, out.sizes, out.strides, out.offset).to_numpy()
    return got, out.to_numpy()


def _inputs(rng, op, n, comp):
    if op in ("asin", "acos"):
        return rng.uniform(-1, 1, n).astype(comp)
    if op in ("sinh", "cosh", "tanh"):
        return rng.uniform(-8, 8, n).astype(comp)
    if op == "log":
        x = np.exp(rng.uniform(-8, 8, n))
    elif op == "exp":
        x = rng.uniform(-9, 9, n)
    else:
        x = rng.uniform(-30, 30, n)
    return x.astype(comp)


def _check_real(got, want, dt):
    comp = REAL[dt]
    g, w = got.astype(np.float64), want.astype(np.float64)
    assert np.array_equal(np.isnan(g), np.isnan(w))
    fin = np.isfinite(w)
    assert np.array_equal(g[~fin & ~np.isnan(w)], w[~fin & ~np.isnan(w)])           # infinities exactly
    ulp = np.spacing(np.abs(want[fin]).astype(comp)).astype(np.float64)
    err = np.abs(g[fin] - w[fin])
    assert np.all(err <= K_ULP[dt] * ulp), (dt, float((err / ulp).max()))


def _check_complex(got, want, dt):
    comp = CPLX[dt]
    mag = np.abs(want.astype(np.complex128))
    fin = np.isfinite(mag)
    ulp = np.spacing(mag[fin].astype(comp)).astype(np.float64)
    for part in (np.real, np.imag):
        err = np.abs(part(got).astype(np.float64)[fin] - part(want).astype(np.float64)[fin])
        assert np.all(err <= K_ULP[dt] * ulp), (dt, float((err / ulp).max()))


@pytest.mark.parametrize("dt", tuple(REAL))
@pytest.mark.parametrize("op", ("sin", "cos", "tan", "exp", "log", "asin", "acos", "atan", "sinh", "cosh", "tanh"))
def test_real_elementary_functions(op, dt):
    rng = rng_for(16000)
    comp = REAL[dt]
    x = _inputs(rng, op, 40000, comp)
    if op == "tan":      # keep away from the poles, where one ulp of the argument moves the value by many
        x = x[np.abs(np.cos(x.astype(np.float64))) > 0.05]
    a = View.from_numpy(x)
    got, want = _run(op, a, View.empty(dt, a.sizes))
    _check_real(got, want, dt)
    # a strided, transposed view goes through the tiled kernel: same values
    m = View.from_numpy(x[: 128 * 96].reshape(128, 96).copy()).permute(1, 0)
    got, want = _run(op, m, View.empty(dt, m.sizes))
    _check_real(got, want, dt)


def _complex_view(z, dt):
    if dt == "chalf":
        pairs = np.stack([z.real, z.imag], axis=-1).astype(np.float16)
        return View(np.ascontiguousarray(pairs).view(np.uint8).reshape(-1).copy(), "chalf", z.shape,
                    tuple(4 * s // z.itemsize for s in z.strides) if z.ndim else (), 0)
    return View.from_numpy(z.astype({"cfloat": np.complex64, "cdouble": np.complex128}[dt]))


@pytest.mark.parametrize("dt", ("cfloat", "cdouble"))
@pytest.mark.parametrize("op", ("sin", "cos", "tan", "exp", "log", "sqrt"))
def test_complex_elementary_functions(op, dt):
    rng = rng_for(16100)
    n = 30000
    z = rng.uniform(-5, 5, n) + 1j * rng.uniform(-5, 5, n)
    if op == "tan":      # away from the poles on the real axis, where the value is ill-conditioned
        z = z[np.abs(np.cos(z)) > 0.1]
    a = _complex_view(z, dt)
    got, want = _run(op, a, View.empty(dt, a.sizes))
    _check_complex(got, want, dt)


def test_special_values_and_branch_cuts():
    x = View.from_numpy(np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, -1.0], dtype=np.float32))
    for op in ("sin", "cos", "exp", "log"):
        got, want = _run(op, x, View.empty("float", x.sizes))
        assert np.array_equal(np.isnan(got), np.isnan(want)), op
        fin = ~np.isnan(want)
        assert np.allclose(got[fin], want[fin], rtol=1e-6, atol=0), (op, got, want)
        assert np.array_equal(np.signbit(got[fin]), np.signbit(want[fin])), op
    z = View.from_numpy(np.array([complex(-1, 0.0), complex(-1, -0.0), complex(-4, 0.0), 0j, complex(0.0, -0.0),
                                  1j, -1j, complex(3, 4)], dtype=np.complex64))
    got, want = _run("sqrt", z, View.empty("cfloat", z.sizes))
    assert np.allclose(got, want, rtol=1e-6, atol=0) and np.array_equal(np.signbit(got.imag), np.signbit(want.imag))
    got, want = _run("log", z.slice(0, 0, 3, 1), View.empty("cfloat", (3,)))
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7) and np.array_equal(np.signbit(got.imag), np.signbit(want.imag))


def _same_class(g, w, rtol):
    """Equal in kind (NaN, infinity with its sign, zero with its sign), else close."""
    if np.isnan(w):
        return bool(np.isnan(g))
    if np.isinf(w) or w == 0:
        return bool(g == w and np.signbit(g) == np.signbit(w))
    return bool(abs(g - w) <= rtol * abs(w))


@pytest.mark.parametrize("dt", ("cfloat", "cdouble"))
def test_complex_functions_of_finite_arguments_with_zero_and_huge_parts(dt):
    # A component that is exactly zero, next to one that makes a factor overflow: the products
    # in sin, cos and exp must give the zero (0 * Inf), not NaN; tiny and huge magnitudes
    # elsewhere.  Every finite argument must agree with the oracle in kind, part by part.
    big = 1e30 if dt == "cfloat" else 1e300
    parts = [0.0, -0.0, 1.0, -1.0, 0.5, big, -big, 1e-40 if dt == "cfloat" else 1e-310, 700.0, -700.0, 89.0, -104.0]
    z = np.array([complex(a, b) for a in parts for b in parts])
    for op in ("sqrt", "exp", "log", "sin", "cos", "tan"):
        a = _complex_view(z, dt)
        got, want = _run(op, a, View.empty(dt, a.sizes))
        rtol = 1e-5 if dt == "cfloat" else 1e-12
        for i in range(len(z)):
            ok = _same_class(got[i].real, want[i].real, rtol) and _same_class(got[i].imag, want[i].imag, rtol)
            assert ok, (op, dt, z[i], got[i], want[i])


def test_complex_square_root_of_infinite_arguments():
    inf, nan = np.inf, np.nan
    z = np.array([complex(a, b) for a in (0.0, -0.0, 1.0, -1.0, inf, -inf, nan) for b in (inf, -inf)] +
                 [complex(a, b) for a in (inf, -inf) for b in (0.0, -0.0, 2.0, -2.0)], dtype=np.complex64)
    a = View.from_numpy(z)
    got, want = _run("sqrt", a, View.empty("cfloat", a.sizes))
    for i in range(len(z)):
        assert _same_class(got[i].real, want[i].real, 1e-6) and _same_class(got[i].imag, want[i].imag, 1e-6), (z[i], got[i], want[i])


@pytest.mark.parametrize("dt", tuple(REAL))
def test_real_functions_at_special_and_extreme_arguments(dt):
    # zeros, infinities, NaN, the largest and smallest magnitudes, arguments around the overflow
    # and underflow of exp, outside the domain of asin, acos and log: same kind of result
    # (NaN, signed infinity, signed zero) as the oracle, close where finite
    ft = REAL[dt]
    fi = np.finfo(ft)
    vals = np.array([0.0, -0.0, 1.0, -1.0, 0.5, -0.5, 2.0, -2.0, np.inf, -np.inf, np.nan, fi.max, -fi.max, fi.tiny,
                     -fi.tiny, fi.tiny / 4, 1e-3, 11.0, -11.0, 89.0, -89.0, 104.0, -104.0, 709.0, 710.0, -745.0,
                     -746.0, 1e4, -1e4, 1.0000001, -1.0000001], dtype=ft)
    rtol = {"half": 2e-3, "float": 1e-5, "double": 1e-12}[dt]
    for op in ("sin", "cos", "tan", "exp", "log", "asin", "acos", "atan", "sinh", "cosh", "tanh", "sqrt"):
        a = View.from_numpy(vals.copy())
        got, want = _run(op, a, View.empty(dt, a.sizes))
        for i in range(len(vals)):
            assert _same_class(float(got[i]), float(want[i]), rtol), (op, dt, float(vals[i]), float(got[i]), float(want[i]))


def test_mixed_types_and_errors():
    import paper_1810_08723_amd as ocn
    rng = rng_for(16200)
    # integer input, floating output: converted on load, evaluated in the output type (generic-dtype kernel)
    i = View.from_numpy(rng.integers(-20, 20, size=(500,), dtype=np.int32))
    got, want = _run("exp", i, View.empty("double", (500,)))
    _check_real(got, want, "double")
    got, want = _run("sin", View.from_numpy(rng.uniform(-3, 3, 300).astype(np.float64)), View.empty("float", (300,)))
    _check_real(got, want, "float")
    dv = H.DeviceViews()
    with pytest.raises(ocn.OcnError) as e:       # no elementary functions in integer arithmetic
        ocn.unary("sin", dv.tensor(i), dv.tensor(View.empty("int32", (500,))))
    assert e.value.code == ocn.binding.ERR["DTYPE"]
