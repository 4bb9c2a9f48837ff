"""GPU parity of reductions: every operation and input type, reduced-fastest / kept-fastest /
general layouts, one and two passes, several axes, empty and degenerate cases."""
import numpy as np
import pytest

import exactmath as X
import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import DTYPES, View

pytestmark = pytest.mark.gpu

_F = {"half": np.float16, "float": np.float32, "double": np.float64,
      "chalf": np.float16, "cfloat": np.float32, "cdouble": np.float64}
# |gpu - oracle| <= REL * sum|x|: the oracle accumulates sequentially in fp64 (compensated for
# double inputs), the GPU in a tree of fp32 (half inputs) or fp64 partial sums
REL = {"half": 1e-3, "float": 1e-6, "double": 1e-13, "chalf": 1e-3, "cfloat": 1e-6, "cdouble": 1e-13}


def _acc_dtype(op, dt):
    if op in ("any", "all"):
        return "bool"
    if op in ("min", "max"):
        return dt
    k = X.kind(dt)
    if k in "bi":
        return "int64"
    if k == "u":
        return "uint64"
    return {"half": "float", "float": "double", "double": "double",
            "chalf": "cfloat", "cfloat": "cdouble", "cdouble": "cdouble"}[dt]


def _check(op, a: View, axes, out_dtype=None):
    out_dtype = out_dtype or _acc_dtype(op, a.dtype)
    kept = [s for d, s in enumerate(a.sizes) if d not in axes]
    out = View.empty(out_dtype, kept)
    got, want = H.run_reduce(op, a, axes, out)
    exact = not (op in ("sum", "prod") and X.kind(a.dtype) in "fc")
    if exact:
        assert H.storages_equal(out_dtype, got, want), (op, a.dtype, axes, H.first_mismatch(out_dtype, got, want))
        return
    comp = _F[out_dtype]
    g = got.view(comp).astype(np.float64)
    w = want.view(comp).astype(np.float64)
    x = a.to_numpy()
    x = x.astype(np.float64) if not np.iscomplexobj(x) else x
    if a.dtype in ("chalf",):
        mag = np.abs(x).sum(axis=tuple(axes)).reshape(-1)          # trailing (re, im) axis kept
    elif X.kind(a.dtype) == "c":
        z = a.to_numpy()
        mag = np.stack([np.abs(z.real).sum(axis=tuple(axes)), np.abs(z.imag).sum(axis=tuple(axes))], axis=-1).reshape(-1)
    else:
        mag = np.abs(x).sum(axis=tuple(axes)).reshape(-1)
    if op == "prod":
        assert np.allclose(g, w, rtol=1e-5 if a.dtype != "double" else 1e-12, atol=0, equal_nan=True)
        return
    rel = max(REL[a.dtype], {"half": 1e-3, "float": 1e-7, "double": 0}.get(out_dtype, 0))  # output rounding
    # overflowed or NaN sums (the mixed-magnitude generator reaches past the half range) must
    # agree in kind; everything finite must agree within the bound
    fin = np.isfinite(w) & np.isfinite(mag)
    assert np.array_equal(np.isnan(g[~fin]), np.isnan(w[~fin])) or not np.isfinite(mag[~fin]).any()
    bound = rel * mag[fin] + 1e-300
    assert np.all(np.abs(g[fin] - w[fin]) <= bound), (op, a.dtype, axes, float(np.abs(g[fin] - w[fin]).max()))


@pytest.mark.parametrize("dt", X.ALL)
def test_all_ops_reduced_axis_fastest(dt):
    rng = rng_for(10000 + X.ALL.index(dt))
    a = random_view(rng, dt, (41, 777), specials=False)
    for op in ("sum", "min", "max", "any", "all"):
        if op in ("min", "max") and X.kind(dt) == "c":
            continue
        print("rows", op, dt, flush=True)
        _check(op, a, [1])


@pytest.mark.parametrize("dt", X.ALL)
def test_all_ops_kept_axis_fastest(dt):
    rng = rng_for(10100 + X.ALL.index(dt))
    a = random_view(rng, dt, (613, 95), specials=False)
    for op in ("sum", "min", "max", "any", "all"):
        if op in ("min", "max") and X.kind(dt) == "c":
            continue
        print("cols", op, dt, flush=True)
        _check(op, a, [0])


@pytest.mark.parametrize("dt", ("int8", "uint8", "int32", "uint64", "half", "float", "double", "cfloat", "bool"))
def test_full_reduction_two_pass(dt):
    rng = rng_for(10200 + X.ALL.index(dt))
    n = (1 << 21) + 12345
    a = random_view(rng, dt, (n,), specials=False)
    for op in ("sum", "max", "any"):
        if op == "max" and X.kind(dt) == "c":
            continue
        print("full", op, dt, flush=True)
        _check(op, a, [0])


def test_prod():
    rng = rng_for(10300)
    x = (1.0 + 0.01 * rng.standard_normal((50, 300))).astype(np.float32)
    _check("prod", View.from_numpy(x), [1])
    _check("prod", View.from_numpy(x.astype(np.float64)), [0])
    i = rng.integers(-3, 4, size=(40, 30)).astype(np.int16)
    _check("prod", View.from_numpy(i), [1])
    _check("prod", View.from_numpy(i), [0, 1])


def test_min_max_nan_and_signed_zero_on_gpu():
    rng = rng_for(10301)
    for dt in ("half", "float", "double"):
        x = rng.standard_normal((64, 500)).astype(DTYPES[dt][1])
        x[3, 17] = np.nan
        x[9, :] = -0.0
        x[9, 250] = 0.0
        x[10, :] = 0.0
        x[10, 7] = -0.0
        x[11, :] = -np.inf
        x[12, :] = np.inf
        x[13, 0] = -np.nan
        v = View.from_numpy(x)
        for op in ("min", "max"):
            _check(op, v, [1])
            _check(op, v, [0])
            _check(op, v, [0, 1])


def test_several_axes_and_strided_inputs():
    rng = rng_for(10302)
    a = random_view(rng, "float", (6, 10, 12, 18), specials=False)
    for axes in ([1, 2], [0, 3], [0, 1, 2, 3], [3], [0], [2, 0], [1, 3]):
        print("axes", axes, flush=True)
        _check("sum", a, axes)
        _check("max", a, axes)
    p = a.permute(2, 0, 3, 1).flip(0).slice(2, 1, 18, 2)
    for axes in ([0], [1, 2], [3], [0, 1, 2, 3]):
        _check("sum", p, axes)
    i = random_view(rng, "int16", (9, 20, 31)).permute(2, 1, 0)
    for axes in ([0], [1], [2], [0, 2]):
        _check("sum", i, axes)
        _check("min", i, axes)


def test_sum_over_flipped_view_equals_sum_over_original_on_gpu():
    rng = rng_for(10303)
    x = View.from_numpy(rng.integers(-1000, 1000, size=(300, 70)).astype(np.int32))
    for v in (x, x.flip(0), x.flip(1), x.flip(0).flip(1)):
        out = View.empty("int64", (70,))
        got, want = H.run_reduce("sum", v, [0], out)
        assert np.array_equal(got, want)
    o1 = View.empty("int64", (70,))
    g1, _ = H.run_reduce("sum", x, [0], o1)
    o2 = View.empty("int64", (70,))
    g2, _ = H.run_reduce("sum", x.flip(0), [0], o2)
    assert np.array_equal(g1, g2)


def test_output_conversion_and_strided_output():
    rng = rng_for(10304)
    a = View.from_numpy(np.full((7, 1000), 100, dtype=np.int8))
    for dt in ("int16", "int32", "uint8", "float", "half", "double", "bool", "cfloat"):
        _check("sum", a, [1], dt)
    f = random_view(rng, "float", (30, 400), specials=False)
    out = View.empty("double", (60,)).slice(0, 1, 60, 2).flip(0)
    got, want = H.run_reduce("sum", f, [1], out)
    assert np.allclose(got.view(np.float64), want.view(np.float64), rtol=1e-12, atol=1e-9)
    sentinel = np.frombuffer(bytes([0xA5] * 8), dtype=np.float64)[0]
    assert np.all(got.view(np.float64)[0::2].view(np.uint64) == np.float64(sentinel).view(np.uint64))


def test_empty_and_degenerate():
    import paper_1810_08723_amd as ocn
    e = View.empty("float", (4, 0))
    for op, dt in (("sum", "float"), ("prod", "float"), ("any", "bool"), ("all", "bool")):
        out = View.empty(dt, (4,))
        got, want = H.run_reduce(op, e, [1], out)
        assert np.array_equal(got, want)
    dv = H.DeviceViews()
    with pytest.raises(ocn.OcnError) as err:
        ocn.reduce("max", dv.tensor(e), [1], dv.tensor(View.empty("float", (4,))))
    assert err.value.code == -10
    rng = rng_for(10305)
    v = random_view(rng, "float", (5, 6), specials=False)
    out = View.empty("float", (5, 6))
    got, want = H.run_reduce("sum", v, [], out)                     # no axes: a cast copy
    assert np.array_equal(got, want)
    one = random_view(rng, "double", (1, 1, 1))
    out = View.empty("double", ())
    got, want = H.run_reduce("max", one, [0, 1, 2], out)
    assert H.storages_equal("double", got, want)


def test_results_are_reproducible_bit_for_bit():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(10306)
    x = rng.standard_normal((2048, 1500)).astype(np.float32)
    dv = H.DeviceViews()
    a = dv.tensor(View.from_numpy(x))
    outs = []
    for _ in range(3):
        o0 = View.empty("float", (1500,))
        o1 = View.empty("float", ())
        t0, t1 = dv.tensor(o0), dv.tensor(o1)
        ocn.reduce("sum", a, [0], t0)
        ocn.reduce("sum", a, [0, 1], t1)
        torch.cuda.synchronize()
        outs.append((dv.download(o0).copy(), dv.download(o1).copy()))
    assert all(np.array_equal(outs[0][0], o[0]) and np.array_equal(outs[0][1], o[1]) for o in outs[1:])


def test_kept_axis_fastest_with_reversed_output():
    # the output walks its fastest axis backwards: the planner must keep the input walking forwards
    rng = rng_for(10307)
    a = random_view(rng, "int16", (3, 10, 122)).permute(0, 2, 1)       # shape (3, 122, 10), axis 1 contiguous
    out = View.empty("int64", (3, 122)).flip(1)
    got, want = H.run_reduce("sum", a, [2], out)
    assert np.array_equal(got, want)
    f = random_view(rng, "float", (300, 257), specials=False)
    out = View.empty("double", (257,)).flip(0)
    got, want = H.run_reduce("sum", f, [0], out)
    assert np.allclose(got.view(np.float64), want.view(np.float64), rtol=1e-12, atol=1e-9)


@pytest.mark.parametrize("row", (1, 2, 3, 4, 7, 16, 33, 64, 100, 129))
def test_short_rows_share_a_wavefront(row):
    # rows shorter than a wavefront's worth of vectors: groups of 1 .. 64 lanes per output,
    # several outputs per wavefront, the last wavefront partly idle
    rng = rng_for(10320 + row)
    for dt in ("float", "int8", "half", "double", "cfloat"):
        a = random_view(rng, dt, (301, row), specials=False)
        plan = H.plan_reduce("sum", a, [1], View.empty(_acc_dtype("sum", dt), (301,)))
        assert plan["kernel"] == ("red_rows" if row > 1 else "red_generic"), plan   # a length-1 axis is dropped
        _check("sum", a, [1])
        if dt not in ("cfloat",):
            _check("max", a, [1])
    # the same rows inside a wider buffer (row stride larger than the row) and misaligned
    wide = random_view(rng, "float", (150, row + 5), specials=False).slice(1, 1, row + 1, 1)
    _check("sum", wide, [1])


def test_reductions_over_strided_axes_are_parallel():
    import paper_1810_08723_amd as ocn
    rng = rng_for(10340)
    # full reduction of an every-other-element view: lanes share the single output
    a = random_view(rng, "float", (200001,), specials=False).slice(0, 0, 200001, 2)
    plan = H.plan_reduce("sum", a, [0], View.empty("double", ()))
    assert plan["kernel"] == "red_rows" and plan["passes"] == 2, plan
    _check("sum", a, [0])
    _check("min", a, [0])
    i8 = random_view(rng, "int8", (99991,)).slice(0, 3, 99991, 3)
    _check("sum", i8, [0])
    # strided along the reduced axis and along the kept axis (no contiguous axis at all)
    b = random_view(rng, "float", (130, 70, 2), specials=False).select(2, 1)
    for axes in ([0], [1], [0, 1]):
        _check("sum", b, axes)
        _check("max", b, axes)
    # kept axis faster than the reduced one, but not contiguous: few outputs, long reduction
    c = random_view(rng, "double", (5000, 12, 2), specials=False).select(2, 0)
    plan = H.plan_reduce("sum", c, [0], View.empty("double", (12,)))
    assert plan["kernel"] == "red_rows", plan
    _check("sum", c, [0])
    # two reduced axes, neither contiguous, permuted
    d = random_view(rng, "int32", (40, 9, 50, 2)).select(3, 1).permute(2, 0, 1)
    for axes in ([0, 1], [1, 2], [0, 2], [0, 1, 2]):
        _check("sum", d, axes)


def test_second_pass_with_few_and_many_partials():
    rng = rng_for(10350)
    # rows split into fewer than 32 parts, and kept-fastest columns split into many
    a = random_view(rng, "float", (3, 300000), specials=False)
    plan = H.plan_reduce("sum", a, [1], View.empty("double", (3,)))
    assert plan["passes"] == 2, plan
    _check("sum", a, [1])
    b = random_view(rng, "float", (40000, 70), specials=False)
    plan = H.plan_reduce("sum", b, [0], View.empty("double", (70,)))
    assert plan["kernel"] == "red_cols" and plan["passes"] == 2 and plan["split"] >= 64, plan
    _check("sum", b, [0])
    _check("max", b, [0])


@pytest.mark.parametrize("ncol", (1, 2, 3, 5, 8, 16, 31, 40, 64, 100))
def test_few_columns_share_a_wavefront(ncol):
    # kept-fastest layouts with fewer column lanes than a wavefront: several rows per wavefront
    rng = rng_for(10360 + ncol)
    for dt in ("float", "int8", "double", "half", "cfloat"):
        a = random_view(rng, dt, (1237, ncol), specials=False)
        if ncol > 1:
            plan = H.plan_reduce("sum", a, [0], View.empty(_acc_dtype("sum", dt), (ncol,)))
            assert plan["kernel"] == "red_cols", plan
        _check("sum", a, [0])
        if dt != "cfloat":
            _check("min", a, [0])
    # more kept dims in front of the columns, and a long reduction that is split
    b = random_view(rng, "float", (7, 50, ncol), specials=False)
    _check("sum", b, [1])
    c = random_view(rng, "int16", (70000, ncol))
    _check("sum", c, [0])


def test_broadcast_inputs():
    # zero strides along reduced and kept axes (views made by broadcasting): every layout branch
    rng = rng_for(10370)
    row = random_view(rng, "int32", (1, 70))
    col = random_view(rng, "int32", (300, 1))
    one = random_view(rng, "float", (1, 1), specials=False)
    for v in (row.broadcast_to((300, 70)), col.broadcast_to((300, 70)), one.broadcast_to((300, 70))):
        for axes in ([0], [1], [0, 1]):
            _check("sum", v, axes)
            _check("max", v, axes)
    cube = random_view(rng, "double", (20, 1, 33), specials=False).broadcast_to((20, 500, 33))
    for axes in ([1], [0, 1], [1, 2], [2], [0, 2], [0, 1, 2]):
        _check("sum", cube, axes)
    wide = random_view(rng, "int8", (1, 5000)).broadcast_to((4000, 5000))     # long reductions of a broadcast axis
    _check("sum", wide, [0])
    _check("sum", wide, [1])
    _check("sum", wide, [0, 1])


@pytest.mark.parametrize("seed", range(12))
def test_fuzz_float_reductions(seed):
    # random shapes, strides (steps, flips, permuted storage, zero strides) and axes with
    # floating types: sums within the tolerance of their type, min/max bit for bit
    from workloads.fuzz import random_shape, random_strided_view
    rng = rng_for(10400 + seed)
    for it in range(8):
        shape = random_shape(rng, max_ndim=5, max_elems=30000)
        if len(shape) == 0 or 0 in shape:
            continue
        dt = ("half", "float", "double", "cfloat")[int(rng.integers(0, 4))]
        a = random_strided_view(rng, dt, shape, specials=False, allow_broadcast=bool(it % 2))
        if tuple(a.sizes) != tuple(shape):
            while a.ndim < len(shape):
                a = a.unsqueeze(0)
            a = a.broadcast_to(shape)
        naxes = int(rng.integers(1, len(shape) + 1))
        axes = sorted(int(x) for x in rng.permutation(len(shape))[:naxes])
        print("fuzz-float-reduce", seed, it, shape, axes, dt, a.strides, flush=True)
        _check("sum", a, axes)
        if dt != "cfloat":
            _check("max", a, axes)


@pytest.mark.parametrize("n", (1, 2, 3, 5, 7, 8, 9, 11, 15, 16, 19))
def test_half_min_max_with_a_partial_last_vector(n):
    # rows whose length is not a multiple of the eight halves of a vector, starting on a
    # 16-byte boundary (the vector path), with subnormals, infinities and signed zeros among
    # the values: the elements of the partial vector must all take part, and only they
    bits = np.array([0xFC00, 0x0008, 0xF442, 0x8000, 0x0000, 0x8001, 0x7BFF, 0x0001, 0x7C00, 0x3C00, 0xBC00],
                    dtype=np.uint16)
    rng = rng_for(10500 + n)
    for trial in range(6):
        row = bits[rng.integers(0, len(bits) - (3 if trial < 3 else 0), size=(4, n))]   # first trials: nothing above 1.0
        x = View.from_numpy(row.view(np.float16))
        for op in ("max", "min"):
            _check(op, x, [1])
            _check(op, x, [0, 1])


@pytest.mark.parametrize("dt", ("int8", "uint8"))
def test_column_sums_of_8_bit_integers_spill_before_overflow(dt):
    # extreme values in every row for more rows than a 16-bit half can hold (the packed
    # accumulation spills every 256 rows), a ragged last column block, and several kept dims
    info = np.iinfo(np.int8 if dt == "int8" else np.uint8)
    rng = rng_for(10600 + (dt == "int8"))
    for fill in (info.min, info.max):
        x = np.full((3000, 80), fill, dtype=info.dtype)
        x[rng.integers(0, 3000, 200), rng.integers(0, 80, 200)] = info.max if fill == info.min else info.min
        _check("sum", View.from_numpy(x), [0])
    y = rng.integers(info.min, info.max, size=(5, 1200, 3, 48), endpoint=True).astype(info.dtype)
    _check("sum", View.from_numpy(y), [1])
    _check("sum", View.from_numpy(y), [0, 1])
    z = rng.integers(info.min, info.max, size=(70001, 16), endpoint=True).astype(info.dtype)
    _check("sum", View.from_numpy(z), [0])
