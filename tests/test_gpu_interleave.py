"""The copy from planes into an output whose fastest axis is a few elements long (channel-first
to channel-last): its own kernel, bit for bit against the oracle's copy."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def _plan(a, out):
    import paper_1810_08723_amd as ocn
    ta = ocn.Tensor(1 << 40, a.dtype, a.sizes, a.strides, a.offset, 0, None, a.byteswapped)
    to = ocn.Tensor(1 << 41, out.dtype, out.sizes, out.strides, out.offset, 0, None, out.byteswapped)
    return ocn.plan_unary("ident", ta, to)


@pytest.mark.parametrize("dtype", ("int8", "half", "float", "double", "cfloat", "int16"))
@pytest.mark.parametrize("c", (2, 3, 4, 5, 7, 8))
def test_planes_to_interleaved(dtype, c):
    rng = rng_for(20000 + c)
    n, h, w = 3, 20, 24            # 480 positions per plane: rows end inside a wavefront
    planes = random_view(rng, dtype, (n, c, h, w))
    a = planes.permute(0, 2, 3, 1)
    out = View.empty(dtype, (n, h, w, c))
    assert _plan(a, out)["kernel"] == "ew_interleave"
    print("interleave", dtype, c, flush=True)
    H.check_unary("ident", a, out)
    # planes in reverse order (a negative plane stride), and both sides in the other byte order
    H.check_unary("ident", planes.flip(1).permute(0, 2, 3, 1), View.empty(dtype, (n, h, w, c)))
    if dtype != "int8":
        af = planes.in_other_byte_order().permute(0, 2, 3, 1)
        of = View.empty(dtype, (n, h, w, c))
        of = View(of.storage, of.dtype, of.sizes, of.strides, of.offset, True)
        assert _plan(af, of)["kernel"] == "ew_interleave"
        H.check_unary("ident", af, of)


def test_shapes_the_kernel_does_not_take_go_elsewhere():
    rng = rng_for(20100)
    planes = random_view(rng, "float", (2, 3, 10, 13))             # 130 positions: not a multiple of 4
    a = planes.permute(0, 2, 3, 1)
    out = View.empty("float", (2, 10, 13, 3))
    assert _plan(a, out)["kernel"] != "ew_interleave"
    H.check_unary("ident", a, out)
    wide = random_view(rng, "float", (2, 3, 8, 16)).permute(0, 2, 3, 1)
    assert _plan(wide, View.empty("double", (2, 8, 16, 3)))["kernel"] != "ew_interleave"   # a cast, not a copy
    H.check_unary("ident", wide, View.empty("double", (2, 8, 16, 3)))


def test_many_workgroups():
    rng = rng_for(20200)
    planes = View.from_numpy(rng.standard_normal((5, 3, 128, 132)).astype(np.float32))
    a = planes.permute(0, 2, 3, 1)
    out = View.empty("float", (5, 128, 132, 3))
    assert _plan(a, out)["kernel"] == "ew_interleave" and _plan(a, out)["grid"] > 64
    H.check_unary("ident", a, out)
