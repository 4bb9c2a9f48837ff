"""Reductions at sizes where every wavefront-sharing form runs many workgroups deep: short rows
(several outputs per wavefront), few columns (several rows per wavefront, split over workgroups,
second pass), a strided full reduction and a reduction over non-adjacent axes.  Whole outputs go
through the oracle where it finishes in seconds, otherwise a sample of the output rows does."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def _gpu_reduce(op, a: View, axes, out: View):
    import torch
    import paper_1810_08723_amd as ocn
    dv = H.DeviceViews()
    ocn.reduce(op, dv.tensor(a), list(axes), dv.tensor(out))
    torch.cuda.synchronize()
    return dv.download(out).copy()


@pytest.mark.parametrize("row", (16, 64, 100))
def test_many_short_rows_sampled(row):
    from oracle import binding as O
    rng = rng_for(18000 + row)
    n = (1 << 20) + 37
    x = rng.standard_normal((n, row), dtype=np.float32)
    a = View.from_numpy(x)
    out = View.empty("float", (n,))
    got = _gpu_reduce("sum", a, [1], out).view(np.float32)
    pick = np.unique(np.concatenate([rng.integers(0, n, size=2000), [0, 1, n - 2, n - 1]]))
    sample = View.from_numpy(np.ascontiguousarray(x[pick]))
    want = View.empty("float", (len(pick),))
    O.reduce("sum", sample, [1], want)
    w = want.storage.view(np.float32).astype(np.float64)
    bound = 1e-6 * np.abs(x[pick].astype(np.float64)).sum(axis=1) + 1e-7 * np.abs(w)
    assert np.all(np.abs(got[pick].astype(np.float64) - w) <= bound)
    # exact check of everything with integers (sums are exact in any order)
    xi = rng.integers(-100, 100, size=(n, row)).astype(np.int8)
    outi = View.empty("int64", (n,))
    goti = _gpu_reduce("sum", View.from_numpy(xi), [1], outi).view(np.int64)
    assert np.array_equal(goti, xi.sum(axis=1, dtype=np.int64))
    gotm = _gpu_reduce("max", View.from_numpy(xi), [1], View.empty("int8", (n,))).view(np.int8)
    assert np.array_equal(gotm, xi.max(axis=1))


@pytest.mark.parametrize("ncol,dt", [(16, "float"), (3, "double"), (256, "int8")])
def test_many_rows_few_columns(ncol, dt):
    from oracle import binding as O
    rng = rng_for(18100 + ncol)
    n = (1 << 21) + 11
    if dt == "int8":
        x = rng.integers(-128, 128, size=(n, ncol)).astype(np.int8)
        got = _gpu_reduce("sum", View.from_numpy(x), [0], View.empty("int64", (ncol,))).view(np.int64)
        assert np.array_equal(got, x.sum(axis=0, dtype=np.int64))
        return
    x = rng.standard_normal((n, ncol)).astype({"float": np.float32, "double": np.float64}[dt])
    a = View.from_numpy(x)
    out = View.empty(dt, (ncol,))
    got = _gpu_reduce("sum", a, [0], out).view(x.dtype).astype(np.float64)
    O.reduce("sum", a, [0], out)                                  # the whole thing: a few seconds
    w = out.storage.view(x.dtype).astype(np.float64)
    rel = 1e-6 if dt == "float" else 1e-13
    assert np.all(np.abs(got - w) <= rel * np.abs(x.astype(np.float64)).sum(axis=0) + (1e-7 if dt == "float" else 0) * np.abs(w))
    gotm = _gpu_reduce("min", a, [0], View.empty(dt, (ncol,))).view(x.dtype)
    assert np.array_equal(gotm, x.min(axis=0))


def test_strided_full_and_non_adjacent_axes():
    from oracle import binding as O
    rng = rng_for(18200)
    x = rng.integers(-1000, 1000, size=((1 << 23) + 5,)).astype(np.int32)
    a = View.from_numpy(x).slice(0, 1, x.size, 3)                 # every third element
    got = _gpu_reduce("sum", a, [0], View.empty("int64", ())).view(np.int64)
    assert got[0] == int(x[1::3].astype(np.int64).sum())
    xf = rng.standard_normal((1 << 23,), dtype=np.float32)
    af = View.from_numpy(xf).slice(0, 0, xf.size, 2)
    out = View.empty("float", ())
    gotf = float(_gpu_reduce("sum", af, [0], out).view(np.float32)[0])
    O.reduce("sum", af, [0], out)
    assert abs(gotf - float(out.storage.view(np.float32)[0])) <= 1e-6 * float(np.abs(xf[::2].astype(np.float64)).sum())
    # axes (0, 2) of a 4-D tensor, exact with integers
    y = rng.integers(-50, 50, size=(40, 96, 48, 128)).astype(np.int16)
    got = _gpu_reduce("sum", View.from_numpy(y), [0, 2], View.empty("int64", (96, 128))).view(np.int64)
    assert np.array_equal(got.reshape(96, 128), y.sum(axis=(0, 2), dtype=np.int64))
