"""GPU parity for tensors stored in the other byte order (section 3.1.3 of the paper): every
kernel family reverses the scalars of a flagged operand on load and of a flagged output on
store, bit for bit as the oracle does, without a pass of its own."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu

MULTI = ("int16", "int32", "int64", "uint16", "uint32", "uint64", "half", "float", "double", "chalf", "cfloat", "cdouble")


def _flagged_out(dtype, sizes):
    v = View.empty(dtype, sizes)
    return View(v.storage, v.dtype, v.sizes, v.strides, v.offset, True)


@pytest.mark.parametrize("dtype", MULTI)
def test_elementwise_kernels_in_either_byte_order(dtype):
    rng = rng_for(18000)
    shape = (67, 130)
    a, b = random_view(rng, dtype, shape), random_view(rng, dtype, shape)
    af, bf = a.in_other_byte_order(), b.in_other_byte_order()
    for x, y, flag_out in ((af, b, False), (a, bf, True), (af, bf, True), (a, b, True)):
        out = _flagged_out(dtype, shape) if flag_out else View.empty(dtype, shape)
        print("rows", dtype, x.byteswapped, y.byteswapped, flag_out, flush=True)
        H.check_binary("add", x, y, out)                                     # rows kernel
    # transposed operand: tiled kernel (general form: clipped tiles)
    bt = random_view(rng, dtype, shape[::-1]).in_other_byte_order().permute(1, 0)
    H.check_binary("sub", af, bt, _flagged_out(dtype, shape))
    # all-vector tiled form: power-of-two extents
    p2 = (128, 256)
    c = random_view(rng, dtype, p2).in_other_byte_order()
    d = random_view(rng, dtype, p2[::-1]).in_other_byte_order().permute(1, 0)
    H.check_binary("mul", c, d, _flagged_out(dtype, p2))
    # 3-D with a broadcast row and a step: the rows kernel's general path
    e = random_view(rng, dtype, (5, 6, 40)).slice(2, 0, 40, 2).in_other_byte_order()
    f = random_view(rng, dtype, (1, 6, 20)).in_other_byte_order().broadcast_to((5, 6, 20))
    H.check_binary("add", e, f, _flagged_out(dtype, (5, 6, 20)))
    # unary, and in place from one byte order to the other
    H.check_unary("neg", af, _flagged_out(dtype, shape))
    g = a.in_other_byte_order()
    native_again = View(g.storage, g.dtype, g.sizes, g.strides, g.offset, False)
    H.check_unary("ident", g, native_again)


def test_casts_and_mixed_types_in_either_byte_order():
    rng = rng_for(18001)
    shape = (41, 77)
    for src, dst in (("double", "int16"), ("int32", "float"), ("half", "double"), ("float", "half"), ("cfloat", "cdouble"),
                     ("uint64", "uint16"), ("int16", "int8"), ("bool", "int32"), ("double", "bool"), ("cdouble", "chalf")):
        a = random_view(rng, src, shape).in_other_byte_order()
        print("cast", src, dst, flush=True)
        H.check_unary("ident", a, _flagged_out(dst, shape))
        H.check_unary("ident", a.permute(1, 0), _flagged_out(dst, shape[::-1]))
    # generic-dtype kernel: a combination without a specialised kernel
    a = random_view(rng, "int16", shape).in_other_byte_order()
    b = random_view(rng, "uint32", shape).in_other_byte_order()
    H.check_binary("add", a, b, _flagged_out("double", shape))
    H.check_binary("lt", a, b, View.empty("bool", shape))
    # specialised mixed pair (converted on load)
    a = random_view(rng, "int32", (64, 256)).in_other_byte_order()
    b = random_view(rng, "float", (1, 256)).in_other_byte_order().broadcast_to((64, 256))
    H.check_binary("mul", a, b, _flagged_out("float", (64, 256)))
    # complex modulus of a flagged tensor
    z = random_view(rng, "cfloat", shape, specials=False).in_other_byte_order()
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = H.DeviceViews()
    out = _flagged_out("float", shape)
    ocn.unary("abs", dv.tensor(z), dv.tensor(out))
    dv.torch.cuda.synchronize()
    got = View(dv.download(out).copy(), "float", out.sizes, out.strides, out.offset, True).to_numpy()
    O.unary("abs", z, out)
    want = out.to_numpy()
    assert np.all(np.abs(got - want) <= 4 * np.spacing(want))


@pytest.mark.parametrize("dtype", ("int16", "int64", "half", "float", "double", "cfloat"))
def test_reductions_in_either_byte_order(dtype):
    rng = rng_for(18002)
    exact = dtype in ("int16", "int64")
    acc_out = {"int16": "int64", "int64": "int64", "half": "float", "float": "double", "double": "double", "cfloat": "cdouble"}[dtype]

    def data(shape):
        if exact:
            return View.from_numpy(rng.integers(-3000, 3000, size=shape).astype({"int16": np.int16, "int64": np.int64}[dtype]))
        if dtype == "cfloat":
            return View.from_numpy((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)).astype(np.complex64))
        return View.from_numpy(rng.standard_normal(shape).astype({"half": np.float16, "float": np.float32, "double": np.float64}[dtype]))

    def check(op, a, axes, out):
        print("reduce", dtype, op, a.sizes, axes, flush=True)
        got, want = H.run_reduce(op, a, axes, out)
        if exact or op in ("max", "min"):
            assert H.storages_equal(out.dtype, got, want, out.byteswapped)
            return
        g = View(got.copy(), out.dtype, out.sizes, out.strides, out.offset, out.byteswapped).to_numpy()
        w = out.to_numpy()
        x = np.abs(a.to_numpy().astype(np.complex128 if dtype == "cfloat" else np.float64)).sum(axis=tuple(axes))
        tol = {"half": 1e-3, "float": 1e-6, "double": 1e-13, "cfloat": 1e-6}[dtype]
        assert np.all(np.abs(g - w) <= tol * x + 1e-300)

    big = data((300, 1500)).in_other_byte_order()
    check("sum", big, [1], _flagged_out(acc_out, (300,)))              # rows, lean form
    check("sum", big, [0], _flagged_out(acc_out, (1500,)))             # columns
    check("sum", big, [0, 1], _flagged_out(acc_out, ()))               # full, split over workgroups (two launches)
    short = data((900, 24)).in_other_byte_order()
    check("sum", short, [1], _flagged_out(acc_out, (900,)))            # short rows
    strided = data((40, 50, 12)).slice(1, 0, 50, 3).in_other_byte_order()
    check("sum", strided, [0, 2], _flagged_out(acc_out, (17,)))        # two reduced dims, a step
    if dtype != "cfloat":
        check("max", big, [1], _flagged_out(dtype, (300,)))
        check("min", big.permute(1, 0), [0], _flagged_out(dtype, (300,)))


def test_reduction_of_an_elementwise_result_in_either_byte_order():
    """An operand in the other byte order makes the one-call form run as its two calls, whose
    kernels reverse on load and on store: integer results bit for bit, floating sums within the
    reduction bound."""
    import paper_1810_08723_amd as ocn
    rng = rng_for(18004)
    ai = View.from_numpy(rng.integers(-3000, 3000, size=(70, 300)).astype(np.int32)).in_other_byte_order()
    bi = View.from_numpy(rng.integers(-3000, 3000, size=(70, 300)).astype(np.int32))
    for axes, kept in (([1], (70,)), ([0], (300,)), ([0, 1], ())):
        out = _flagged_out("int64", kept)
        dv = H.DeviceViews()
        plan = ocn.plan_binary_reduce("mul", "sum", dv.tensor(ai), dv.tensor(bi), axes, dv.tensor(out), "int32")
        assert not plan["fused"]
        got, want = H.run_binary_reduce("mul", "sum", ai, bi, axes, out, "int32")
        assert H.storages_equal("int64", got, want, out.byteswapped)
        got, want = H.run_binary_reduce("gt", "sum", bi, ai, axes, View.empty("int64", kept), "bool")
        assert H.storages_equal("int64", got, want)
    af = View.from_numpy(rng.standard_normal((70, 300)).astype(np.float32)).in_other_byte_order()
    bf = View.from_numpy(rng.standard_normal((70, 300)).astype(np.float32)).in_other_byte_order()
    out = _flagged_out("float", (70,))
    got, want = H.run_binary_reduce("mul", "sum", af, bf, [1], out, "float")
    g = View(got.copy(), "float", out.sizes, out.strides, out.offset, out.byteswapped).to_numpy()
    w = out.to_numpy()
    mag = np.abs(af.to_numpy().astype(np.float64) * bf.to_numpy().astype(np.float64)).sum(axis=1)
    assert np.all(np.abs(g - w) <= 1e-6 * mag + 1e-300)


@pytest.mark.parametrize("dt", ("int16", "float", "double", "chalf", "cfloat", "cdouble"))
def test_gather_and_scatter_between_byte_orders(dt):
    """Indexed copies between tensors stored in different byte orders move values: single
    elements (four offsets per lane, ragged counts, an unaligned rows side) and rows of 16-byte
    pieces, in both directions."""
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import indexing as OI
    from workloads.views import itemsize
    es = itemsize(dt)
    rng = rng_for(18005 + es)
    dev64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).to("cuda:0")
    for src_swapped, out_swapped in ((True, False), (False, True), (True, True)):
        src = random_view(rng, dt, (3000,))
        if src_swapped:
            src = src.in_other_byte_order()
        scalar = View(src.storage, dt, (), (), 0, src.byteswapped)
        for n, skew in ((1, 0), (7, 0), (1024, 0), (1027, 1)):
            offs = rng.integers(0, 3000, size=n).astype(np.int64) * es
            base = View.empty(dt, (n + skew,))
            out = View(base.storage, dt, (n,), (es,), skew * es, out_swapped)
            dv = H.DeviceViews()
            ocn.gather(dv.tensor(scalar), dev64(offs), 0, 2999 * es, dv.tensor(out))
            torch.cuda.synchronize()
            got = dv.download(out).copy()
            OI.gather(scalar, offs, out, 0, 2999 * es)
            assert np.array_equal(got, out.storage), (dt, n, skew, src_swapped, out_swapped)
            perm = rng.permutation(3000)[:n].astype(np.int64) * es
            vals_base = random_view(rng, dt, (n + skew,))
            vals = View(vals_base.storage, dt, (n,), (es,), skew * es, out_swapped)
            target = random_view(rng, dt, (3000,))
            tscalar = View(target.storage, dt, (), (), 0, src_swapped)
            dv = H.DeviceViews()
            ocn.scatter(dv.tensor(vals), dev64(perm), 0, 2999 * es, dv.tensor(tscalar))
            torch.cuda.synchronize()
            got_t = dv.download(tscalar).copy()
            OI.scatter(vals, perm, tscalar, 0, 2999 * es)
            assert np.array_equal(got_t, target.storage), (dt, n, skew, src_swapped, out_swapped)
        # rows of several elements (16-byte pieces where the offsets allow)
        table = random_view(rng, dt, (200, 24))
        if src_swapped:
            table = table.in_other_byte_order()
        inner = View(table.storage, dt, (24,), (es,), 0, table.byteswapped)
        roffs = rng.integers(0, 200, size=77).astype(np.int64) * 24 * es
        rows_base = View.empty(dt, (77, 24))
        rows = View(rows_base.storage, dt, (77, 24), rows_base.strides, 0, out_swapped)
        dv = H.DeviceViews()
        ocn.gather(dv.tensor(inner), dev64(roffs), 0, 199 * 24 * es, dv.tensor(rows))
        torch.cuda.synchronize()
        got = dv.download(rows).copy()
        OI.gather(inner, roffs, rows, 0, 199 * 24 * es)
        assert np.array_equal(got, rows.storage), (dt, "rows", src_swapped, out_swapped)


def test_calls_that_take_native_order_only_say_so():
    import paper_1810_08723_amd as ocn
    rng = rng_for(18003)
    import torch
    idx = View.from_numpy(rng.integers(0, 8, size=(8,)).astype(np.int64)).in_other_byte_order()
    dv = H.DeviceViews()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    with pytest.raises(ocn.OcnError) as e:      # index arrays are the library's own native data
        ocn.index_offsets(dv.tensor(idx), 8, 4, dv.tensor(View.empty("int64", (8,))), bad)
    assert e.value.code == ocn.binding.ERR["BYTEORDER"]
    # one-byte scalars have no byte order: the flag is ignored
    m = random_view(rng, "int8", (8, 8)).in_other_byte_order()
    n = random_view(rng, "int8", (8, 8))
    H.check_binary("add", m, n, View.empty("int8", (8, 8)))
    got, want = H.run_binary_reduce("mul", "sum", m, n, [1], View.empty("int64", (8,)), "int8")
    assert np.array_equal(got, want)
