"""GPU parity of the byte-swap operation and of the domain check behind the compute modes."""
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
