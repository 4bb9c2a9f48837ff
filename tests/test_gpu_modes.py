"""GPU parity of the byte-swap operation, of the domain check behind the compute modes, and of
the compute modes themselves (standard, warning, error, complex)."""
import numpy as np
import pytest

import gpu_harness as H
from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", ("int8", "uint8", "int16", "uint16", "int32", "uint32", "int64", "uint64", "bool"))
def test_byte_swap(dt):
    rng = rng_for(18000)
    a = random_view(rng, dt, (67, 130))
    H.check_unary("bswap", a, View.empty(dt, (67, 130)))                    # rows kernel
    H.check_unary("bswap", a.permute(1, 0), View.empty(dt, (130, 67)))      # tiled kernel
    H.check_unary("bswap", a, a)                                            # in place


def test_float_data_in_the_other_byte_order():
    import paper_1810_08723_amd as ocn
    rng = rng_for(18001)
    x = rng.standard_normal((50, 40)).astype(np.float64)
    foreign = View.from_numpy(x.byteswap().view(np.uint64))                  # the bytes as another machine wrote them
    native = View.empty("uint64", (50, 40))
    dv = H.DeviceViews()
    ocn.unary("bswap", dv.tensor(foreign), dv.tensor(native))
    dv.torch.cuda.synchronize()
    assert np.array_equal(dv.download(native).view(np.float64).reshape(50, 40), x)


@pytest.mark.parametrize("dt", ("float", "double", "half", "int32", "int8"))
def test_domain_check(dt):
    import paper_1810_08723_amd as ocn
    rng = rng_for(18100)
    npdt = {"float": np.float32, "double": np.float64, "half": np.float16, "int32": np.int32, "int8": np.int8}[dt]
    x = np.abs(rng.standard_normal((300, 257)) * 20).astype(npdt)
    for plant in (None, (0, 0), (299, 256), (123, 45)):
        y = x.copy()
        if plant is not None:
            y[plant] = -1
        for view in (View.from_numpy(y), View.from_numpy(y).permute(1, 0), View.from_numpy(y).slice(1, 1, 257, 2)):
            dv = H.DeviceViews()
            for op in ("sqrt", "log", "exp", "neg"):
                flag = ocn.domain_check(op, dv.tensor(view))
                dv.torch.cuda.synchronize()
                assert bool(flag.cpu()[0]) == O.domain_check(op, view), (dt, plant, op, view.strides)
    # NaN, zeros and +Inf are inside the domain; -Inf is not
    if dt in ("float", "double"):
        z = View.from_numpy(np.array([0.0, -0.0, np.nan, np.inf], dtype=npdt))
        dv = H.DeviceViews()
        assert not bool(ocn.domain_check("sqrt", dv.tensor(z)).cpu()[0])
        w = View.from_numpy(np.array([1.0, -np.inf], dtype=npdt))
        assert bool(ocn.domain_check("log", H.DeviceViews().tensor(w)).cpu()[0])


@pytest.mark.parametrize("dt", ("float", "double", "half", "int16"))
def test_domain_check_of_inverse_sine_and_cosine(dt):
    import paper_1810_08723_amd as ocn
    rng = rng_for(18200)
    npdt = {"float": np.float32, "double": np.float64, "half": np.float16, "int16": np.int16}[dt]
    x = (rng.uniform(-1, 1, (200, 130)) if dt != "int16" else rng.integers(-1, 2, (200, 130))).astype(npdt)
    for plant in (None, (0, 0), (199, 129)):
        y = x.copy()
        if plant is not None:
            y[plant] = npdt(2) if dt == "int16" else np.nextafter(npdt(1), npdt(2))
        for view in (View.from_numpy(y), View.from_numpy(y).permute(1, 0)):
            dv = H.DeviceViews()
            for op in ("asin", "acos", "atan", "cosh"):
                flag = ocn.domain_check(op, dv.tensor(view))
                dv.torch.cuda.synchronize()
                assert bool(flag.cpu()[0]) == O.domain_check(op, view), (dt, plant, op)


def test_domain_check_on_complex_is_always_clear():
    import paper_1810_08723_amd as ocn
    z = View.from_numpy(np.array([-1 + 0j, -2 - 3j], dtype=np.complex64))
    flag = ocn.domain_check("sqrt", H.DeviceViews().tensor(z))
    assert not bool(flag.cpu()[0])


def _mode_case(op, x, cdt="cdouble"):
    a = View.from_numpy(np.asarray(x, dtype=np.float64))
    return a, View.empty("double", a.sizes), View.empty(cdt, a.sizes)


@pytest.mark.parametrize("op", ("sqrt", "log", "acos", "asin", "sin"))
def test_compute_modes_follow_the_oracle(op):
    # standard / warning / error / complex (section 3.2.1) on inputs inside and outside the
    # operator's domain: the same answer to "outside?", the same output written, the same
    # values (ulp class), and an untouched output where error mode refuses
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    rng = rng_for(15100)
    inside = {"sqrt": rng.uniform(0, 9, 5000), "log": rng.uniform(0.01, 9, 5000), "acos": rng.uniform(-1, 1, 5000),
              "asin": rng.uniform(-1, 1, 5000), "sin": rng.uniform(-9, 9, 5000)}[op]
    outside = inside.copy()
    outside[1234] = -2.5
    for x in (inside, outside):
        for mode in O.MODES:
            a, out, outc = _mode_case(op, x)
            dv = H.DeviceViews()
            ta, to, tc = dv.tensor(a), dv.tensor(out), dv.tensor(outc)
            print(op, mode, "outside" if x is outside else "inside", flush=True)
            try:
                got = ocn.unary_mode(op, mode, ta, to, tc)
            except ocn.OcnError as e:
                assert e.code == ocn.binding.ERR["DOMAIN"]
                got = "refused"
            dv.torch.cuda.synchronize()
            g_out, g_outc = dv.download(out).copy(), dv.download(outc).copy()
            try:
                want = O.unary_mode(op, mode, a, out, outc)
            except O.DomainError:
                want = "refused"
            assert got == want, (op, mode, got, want)
            if want == "refused":
                assert np.all(g_out == 0xA5) and np.all(g_outc == 0xA5)       # nothing was written
                continue
            if want["wrote"] == "out":
                g, w = g_out.view(np.float64), out.to_numpy()
                assert np.all(g_outc == 0xA5)
                assert np.array_equal(np.isnan(g), np.isnan(w))
                ok = ~np.isnan(w)
                assert np.all(np.abs(g[ok] - w[ok]) <= 4 * np.spacing(np.abs(w[ok])))
            else:
                g, w = g_outc.view(np.complex128), outc.to_numpy()
                assert np.all(g_out == 0xA5)
                mag = np.abs(w)
                for part in (np.real, np.imag):
                    assert np.all(np.abs(part(g) - part(w)) <= 8 * np.spacing(mag))


def test_compute_mode_errors_come_before_any_launch():
    import paper_1810_08723_amd as ocn
    a, out, outc = _mode_case("sqrt", [1.0, -1.0, 4.0])
    dv = H.DeviceViews()
    ta, to, tc = dv.tensor(a), dv.tensor(out), dv.tensor(outc)
    with pytest.raises(ocn.OcnError) as e:        # complex mode needs a complex second output
        ocn.unary_mode("sqrt", "complex", ta, to, to)
    assert e.value.code == ocn.binding.ERR["DTYPE"]
    with pytest.raises(ocn.OcnError) as e:
        ocn.unary_mode("sqrt", "complex", ta, to, None)
    assert e.value.code == ocn.binding.ERR["NULLPTR"]
    bad = ocn.Tensor(to.base, "double", (4,), (8,), 0, 0, to.keepalive)       # shape mismatch
    with pytest.raises(ocn.OcnError) as e:
        ocn.unary_mode("sqrt", "warning", ta, bad, tc)
    assert e.value.code == ocn.binding.ERR["SHAPE"]
    dv.torch.cuda.synchronize()
    assert np.all(dv.download(out) == 0xA5) and np.all(dv.download(outc) == 0xA5)
