"""Elementwise layouts at sizes of many tiles per XCD, whole outputs against the oracle:
widening and narrowing casts of transposed views, channel-last <-> channel-first copies, a
transpose with odd extents, mixed-type arithmetic with a transposed operand, and the 5-D
permutation of the benchmark at a quarter of its size (tiles paired on an XCD)."""
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("din,dout", [("int8", "int32"), ("half", "float"), ("float", "double"),
                                      ("double", "float"), ("float", "half"), ("int32", "int8")])
def test_casts_of_transposed_views(din, dout):
    rng = rng_for(19000 + sum(map(ord, din + dout)))
    a = random_view(rng, din, (2048, 3072)).permute(1, 0)
    H.check_unary("ident", a, View.empty(dout, (3072, 2048)))


@pytest.mark.parametrize("c", (3, 4, 8))
def test_channel_last_and_channel_first(c):
    rng = rng_for(19100 + c)
    nhwc = random_view(rng, "float", (8, 192, 160, c), specials=False)
    H.check_unary("ident", nhwc.permute(0, 3, 1, 2), View.empty("float", (8, c, 192, 160)))
    nchw = random_view(rng, "float", (8, c, 192, 160), specials=False)
    H.check_unary("neg", nchw.permute(0, 2, 3, 1), View.empty("float", (8, 192, 160, c)))
    u8 = random_view(rng, "uint8", (16, 200, 120, c))
    H.check_unary("ident", u8.permute(0, 3, 1, 2), View.empty("uint8", (16, c, 200, 120)))


def test_odd_transpose_and_mixed_types():
    rng = rng_for(19200)
    a = random_view(rng, "float", (2003, 3001), specials=False).permute(1, 0)
    b = random_view(rng, "float", (3001, 2003), specials=False)
    H.check_binary("add", a, b, View.empty("float", (3001, 2003)))
    x = random_view(rng, "float", (2048, 1024), specials=False)
    z = random_view(rng, "cfloat", (1024, 2048), specials=False).permute(1, 0)
    H.check_binary("mul", x, z, View.empty("cfloat", (2048, 1024)))
    h = random_view(rng, "half", (1024, 4096), specials=False).permute(1, 0)
    f = random_view(rng, "float", (4096, 1024), specials=False)
    H.check_binary("sub", h, f, View.empty("float", (4096, 1024)))


def test_five_dimensional_permutation_with_paired_tiles():
    import paper_1810_08723_amd as ocn
    from workloads import configs
    cases = configs.config5(shape=(16, 32, 64, 16, 8)) + configs.config5(shape=(16, 32, 64, 16, 8), reading="R2")
    for c in cases:
        dv = H.DeviceViews()
        plan = ocn.plan_binary(c.op, dv.tensor(c.inputs[0]), dv.tensor(c.inputs[1]), dv.tensor(c.out))
        print(c.name, plan["kernel"], plan["unclipped"], plan["tile_group"], flush=True)
        H.check_binary(c.op, c.inputs[0], c.inputs[1], c.out)


@pytest.mark.parametrize("dt", ("int8", "uint8", "bool"))
def test_one_byte_transposes(dt):
    """One-byte elements (sixteen per vector): transposes with extents that are and are not
    multiples of the tile, with a second operand, and with a third tiled axis."""
    rng = rng_for(19400 + len(dt))
    a = random_view(rng, dt, (1024, 1536)).permute(1, 0)
    H.check_unary("ident", a, View.empty(dt, (1536, 1024)))
    if dt != "bool":
        b = random_view(rng, dt, (1536, 1024))
        H.check_binary("add", a, b, View.empty(dt, (1536, 1024)))
        H.check_unary("neg", random_view(rng, dt, (640, 1000)).permute(1, 0), View.empty(dt, (1000, 640)))
    else:
        b = random_view(rng, dt, (1536, 1024))
        H.check_binary("lxor", a, b, View.empty(dt, (1536, 1024)))
    c = random_view(rng, dt, (256, 384, 128)).permute(2, 0, 1)
    H.check_unary("ident", c, View.empty(dt, (128, 256, 384)))
