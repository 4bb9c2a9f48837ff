"""Work that needs more workgroups than one launch may have: the generic-dtype elementwise
kernel, the generic reductions and the index binding loop inside the kernel, gather and scatter
go out in several launches.  Exercised at small sizes by lowering the bound
(ocn_set_max_launch_blocks), and once past the real limit of 2^32 lanes on the cheapest type."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


@pytest.fixture
def few_blocks():
    import paper_1810_08723_amd as ocn
    ocn.binding.set_max_launch_blocks(3)
    yield 3
    ocn.binding.set_max_launch_blocks(0)


def test_generic_dtype_kernel_loops(few_blocks):
    import paper_1810_08723_amd as ocn
    rng = rng_for(19000)
    a = random_view(rng, "int16", (37, 211))
    b = random_view(rng, "uint32", (37, 211))
    ta = ocn.Tensor(1 << 40, "int16", a.sizes, a.strides, 0, 0)
    tb = ocn.Tensor(1 << 41, "uint32", b.sizes, b.strides, 0, 0)
    to = ocn.Tensor(1 << 42, "double", (37, 211), (211 * 8, 8), 0, 0)
    plan = ocn.plan_binary("add", ta, tb, to)
    assert plan["kernel"] == "ew_generic" and plan["grid"] == 3            # 31 workgroups' worth of elements
    H.check_binary("add", a, b, View.empty("double", (37, 211)))
    H.check_binary("add", a.permute(1, 0), b.permute(1, 0), View.empty("double", (211, 37)))
    # a specialised contiguous operation too large for the bound goes to the looping kernel
    x = random_view(rng, "float", (5000,))
    tx = ocn.Tensor(1 << 40, "float", (5000,), (4,), 0, 0)
    assert ocn.plan_unary("neg", tx, ocn.Tensor(1 << 41, "float", (5000,), (4,), 0, 0))["kernel"] == "ew_generic"
    H.check_unary("neg", x, View.empty("float", (5000,)))


def test_reductions_fall_back_to_the_looping_kernel(few_blocks):
    rng = rng_for(19001)
    x = View.from_numpy(rng.integers(-100, 100, size=(3000, 40)).astype(np.int32))
    plan = H.plan_reduce("sum", x, [1], View.empty("int64", (3000,)))
    assert plan["kernel"] == "red_generic" and plan["grid"] == 3
    got, want = H.run_reduce("sum", x, [1], View.empty("int64", (3000,)))
    assert np.array_equal(got, want)
    got, want = H.run_reduce("max", x, [0], View.empty("int32", (40,)))
    assert np.array_equal(got, want)


def test_index_binding_gather_and_scatter_in_several_launches(few_blocks):
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import indexing as OI
    rng = rng_for(19002)
    n, dim = 5000, 977
    idx_h = rng.integers(-dim - 3, dim + 3, size=n).astype(np.int64)
    idx = View.from_numpy(idx_h)
    offs = View.empty("int64", (n,))
    dv = H.DeviceViews()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    ocn.index_offsets(dv.tensor(idx), dim, 12, dv.tensor(offs), bad)
    torch.cuda.synchronize()
    want_offs, want_bad = OI.index_offsets(idx_h, dim, 12)
    assert np.array_equal(dv.download(offs).view(np.int64), want_offs) and int(bad.cpu()[0]) == want_bad
    # gather rows of 3 floats (short rows share a workgroup) and rows of 700 (several workgroups a row)
    for inner_n in (3, 700):
        src_h = rng.standard_normal((dim, inner_n)).astype(np.float32)
        src = torch.from_numpy(src_h).to("cuda:0")
        pick = rng.integers(0, dim, size=n).astype(np.int64)
        o = torch.from_numpy(pick * inner_n * 4).to("cuda:0")
        out = torch.full((n, inner_n), -7.0, dtype=torch.float32, device="cuda:0")
        ti = ocn.Tensor(src.data_ptr(), "float", (inner_n,), (4,), 0, 0, src)
        trows = ocn.Tensor(out.data_ptr(), "float", (n, inner_n), (inner_n * 4, 4), 0, 0, out)
        ocn.gather(ti, o, 0, (dim - 1) * inner_n * 4, trows)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), src_h[pick])
        # scatter them back into a fresh tensor through a permutation
        perm = rng.permutation(dim)[:min(n, dim)].astype(np.int64)
        vals = torch.from_numpy(src_h[: len(perm)].copy()).to("cuda:0")
        dst = torch.zeros((dim, inner_n), dtype=torch.float32, device="cuda:0")
        po = torch.from_numpy(perm * inner_n * 4).to("cuda:0")
        tv = ocn.Tensor(vals.data_ptr(), "float", (len(perm), inner_n), (inner_n * 4, 4), 0, 0, vals)
        td = ocn.Tensor(dst.data_ptr(), "float", (inner_n,), (4,), 0, 0, dst)
        ocn.scatter(tv, po, 0, (dim - 1) * inner_n * 4, td)
        torch.cuda.synchronize()
        want = np.zeros((dim, inner_n), dtype=np.float32)
        want[perm] = src_h[: len(perm)]
        assert np.array_equal(dst.cpu().numpy(), want)


def test_generic_dtype_kernel_past_two_to_the_32_lanes():
    # int8 + uint8 -> int8 has no specialised kernel; 2^32 + 2^16 output elements, both inputs
    # broadcast so that only the output is large.  Every row of the output must equal the one
    # row the oracle computes; compared on the device (the comparison is not the engine's work).
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    rows, cols = (1 << 16) + 1, 1 << 16
    rng = rng_for(19003)
    b_h = rng.integers(0, 255, size=cols, endpoint=True).astype(np.uint8)
    a = View.from_numpy(np.array(-5, dtype=np.int8))
    b = View.from_numpy(b_h)
    want = View.empty("int8", (cols,))
    O.binary("add", a, b, want)
    da = torch.from_numpy(a.storage.copy()).to("cuda:0")
    db = torch.from_numpy(b.storage.copy()).to("cuda:0")
    out = torch.full((rows * cols,), 0x5A, dtype=torch.uint8, device="cuda:0")
    ta = ocn.Tensor(da.data_ptr(), "int8", (), (), 0, 0, da)
    tb = ocn.Tensor(db.data_ptr(), "uint8", (cols,), (1,), 0, 0, db)
    to = ocn.Tensor(out.data_ptr(), "int8", (rows, cols), (cols, 1), 0, 0, out)
    plan = ocn.plan_binary("add", ta, tb, to)
    assert plan["kernel"] == "ew_generic" and plan["grid"] == (1 << 24) - 1 and rows * cols > 1 << 32
    print("launching", rows * cols, "elements", flush=True)
    ocn.binary("add", ta, tb, to)
    torch.cuda.synchronize()
    expect = torch.from_numpy(want.storage.copy()).to("cuda:0")
    assert bool((out.view(rows, cols) == expect.unsqueeze(0)).all())
