"""Host planner: dimension canonicalisation (drop, flip, sort, merge - section 4 of the paper)
must not change which addresses belong together, and the worked plans of the benchmark
configurations come out as derived by hand."""
import itertools

import numpy as np
import pytest

import paper_1810_08723_amd as ocn
from workloads import configs
from workloads.fuzz import random_shape, random_strided_view
from workloads.values import rng_for
from workloads.views import View, itemsize

BASES = (0x1000000000, 0x2000000000, 0x3000000000)  # fake, aligned, far apart: never dereferenced


def fake(view: View, which: int) -> ocn.Tensor:
    return ocn.Tensor(BASES[which], view.dtype, view.sizes, view.strides, view.offset, 0)


def raw_address_tuples(a: View, b: View, out: View):
    """(out, a, b) byte offsets for every output index, straight from the raw descriptors."""
    la, lb = out.ndim - a.ndim, out.ndim - b.ndim
    res = []
    for idx in itertools.product(*[range(s) for s in out.sizes]):
        oo = out.offset + sum(i * s for i, s in zip(idx, out.strides))
        ao = a.offset + sum((0 if a.sizes[d] == 1 else idx[la + d]) * a.strides[d] for d in range(a.ndim))
        bo = b.offset + sum((0 if b.sizes[d] == 1 else idx[lb + d]) * b.strides[d] for d in range(b.ndim))
        res.append((oo, ao, bo))
    return sorted(res)


def plan_address_tuples(plan):
    res = []
    for idx in itertools.product(*[range(s) for s in plan["size"]]):
        res.append((plan["offset_out"] + sum(i * s for i, s in zip(idx, plan["stride_out"])),
                    plan["offset_a"] + sum(i * s for i, s in zip(idx, plan["stride_a"])),
                    plan["offset_b"] + sum(i * s for i, s in zip(idx, plan["stride_b"]))))
    return sorted(res)


@pytest.mark.parametrize("seed", range(60))
def test_canonical_plan_preserves_address_tuples(seed):
    rng = rng_for(7000 + seed)
    for _ in range(6):
        shape = random_shape(rng, max_ndim=6, max_elems=700)
        dt = ["uint8", "int16", "float", "double", "cfloat"][int(rng.integers(0, 5))]
        a = random_strided_view(rng, dt, shape, specials=False)
        b = random_strided_view(rng, dt, shape, specials=False)
        out = random_strided_view(rng, dt, shape, writable=True)
        plan = ocn.plan_binary("add", fake(a, 0), fake(b, 1), fake(out, 2))
        if out.numel == 0:
            assert plan["kernel"] == "none"
            continue
        assert plan_address_tuples(plan) == raw_address_tuples(a, b, out)
        # canonical form: output strides positive and sorted, no size-1 dims (unless a single element)
        so = plan["stride_out"]
        assert all(s > 0 for s in so) and list(so) == sorted(so, reverse=True)
        assert all(s > 1 for s in plan["size"]) or out.numel == 1
        # no adjacent pair left that every operand could walk as one dim
        for d in range(plan["ndim"] - 1):
            n = plan["size"][d + 1]
            assert not all(plan[k][d] == plan[k][d + 1] * n for k in ("stride_out", "stride_a", "stride_b"))


def test_worked_plan_config1_is_a_2d_transpose():
    c = configs.config1(1)
    plan = ocn.plan_binary("add", fake(c.inputs[0], 0), fake(c.inputs[1], 1), fake(c.out, 2))
    # dims (0,1) merge for all three operands: [3072, 32], A/C strides (32,1), B strides (1,3072) elements
    assert plan["size"] == (3072, 32)
    assert plan["stride_out"] == (128, 4) and plan["stride_a"] == (128, 4) and plan["stride_b"] == (4, 12288)
    assert plan["kernel"] == "ew_tiled" and plan["stage_b"] and not plan["stage_a"]


def test_worked_plan_config2_keeps_the_flipped_rows():
    c = configs.config2(64, 48)
    plan = ocn.plan_unary("ident", fake(c.inputs[0], 0), fake(c.out, 2))
    # -row_pitch != +8 * cols, so the two dims cannot merge; the source offset sits on the last row
    assert plan["size"] == (64, 48)
    assert plan["stride_a"] == (-48 * 8, 8) and plan["stride_out"] == (96, 2)
    assert plan["offset_a"] == 63 * 48 * 8
    # the widest operand (the double input) moves 16 bytes per lane: two elements
    assert plan["kernel"] == "ew_rows" and plan["vec"] == 2


def test_worked_plan_config3_broadcast_row_blocks_the_merge():
    c = configs.config3(32, 256)
    plan = ocn.plan_binary("mul", fake(c.inputs[0], 0), fake(c.inputs[1], 1), fake(c.out, 2))
    assert plan["size"] == (32, 256) and plan["stride_b"] == (0, 4)
    assert plan["kernel"] == "ew_rows" and plan["compute_dtype"] == "float" and plan["specialised"]


def test_contiguous_operands_flatten_to_one_dimension():
    a = View.empty("float", (7, 5, 3, 11))
    plan = ocn.plan_binary("add", fake(a, 0), fake(a.fresh_copy(), 1), fake(a.fresh_copy(), 2))
    assert plan["size"] == (7 * 5 * 3 * 11,) and plan["kernel"] == "ew_rows"
    # column-major data flattens just the same (axes are sorted by stride first)
    f = View.empty("float", (7, 5, 3, 11), order="F")
    plan = ocn.plan_binary("add", fake(f, 0), fake(f.fresh_copy(), 1), fake(f.fresh_copy(), 2))
    assert plan["size"] == (7 * 5 * 3 * 11,)


def test_worked_plan_config5_stays_five_dimensional():
    cs = configs.config5()
    c = cs[0]
    plan = ocn.plan_binary("mul", fake(c.inputs[0], 0), fake(c.inputs[1], 1), fake(c.out, 2))
    # canonical order = output strides descending: original axes (1, 3, 4, 0, 2); nothing merges
    assert plan["size"] == (32, 64, 8, 16, 64)
    es = 8
    assert plan["stride_out"] == tuple(es * s for s in (524288, 8192, 1024, 64, 1))
    assert plan["stride_a"] == tuple(es * s for s in (1024, 16, 32768, 1, 524288))
    assert plan["stride_b"] == tuple(es * s for s in (32768, 8, 1, 1048576, 512))
    assert plan["kernel"] == "ew_tiled" and plan["stage_a"] and plan["stage_b"]
    assert plan["lds_bytes"] <= 64 * 1024


def test_worked_plan_config5_second_reading():
    # buffers that store the logical dims in permuted order: another stride vector, same plan kind
    c = configs.config5(reading="R2")[0]
    es = 8
    assert c.inputs[0].strides == tuple(es * s for s in (2048, 1, 65536, 32, 4194304))
    assert c.out.strides == tuple(es * s for s in (16384, 64, 1, 262144, 2048))
    plan = ocn.plan_binary("mul", fake(c.inputs[0], 0), fake(c.inputs[1], 1), fake(c.out, 2))
    # canonical order = original axes (3, 0, 4, 1, 2); no pair merges for all three operands
    assert plan["size"] == (64, 16, 8, 32, 64)
    assert plan["stride_out"] == tuple(es * s for s in (262144, 16384, 2048, 64, 1))
    assert plan["stride_a"] == tuple(es * s for s in (32, 2048, 4194304, 1, 65536))
    assert plan["stride_b"] == tuple(es * s for s in (8, 1048576, 1, 32768, 512))
    assert plan["kernel"] == "ew_tiled" and plan["stage_a"] and plan["stage_b"]


def test_unclipped_form_and_staging_budget():
    # configuration 1 (a pure transpose of power-of-two extents) and configuration 5 take the
    # lean form of the tiled kernel.  Tiles grow to full-line runs within 32 KiB of LDS and
    # beyond that only until each of the 256 lanes has a whole vector in every order.
    c1 = configs.config1(8)
    plan = ocn.plan_binary("add", fake(c1.inputs[0], 0), fake(c1.inputs[1], 1), fake(c1.out, 2))
    assert plan["kernel"] == "ew_tiled" and plan["unclipped"]
    assert plan["tile_log2"] == (5, 5) and plan["lds_bytes"] == 4 * 1024   # 128 B runs both ways
    for c in configs.config5() + configs.config5(reading="R2"):
        plan = ocn.plan_binary(c.op, fake(c.inputs[0], 0), fake(c.inputs[1], 1), fake(c.out, 2))
        assert plan["kernel"] == "ew_tiled" and plan["unclipped"], c.name
        if plan["stage_a"] and plan["stage_b"]:
            # three different fastest axes: 16 elements (128 B) along the output's and a's,
            # 8 (all there is) along b's
            assert plan["lds_bytes"] == 32 * 1024 and sorted(plan["tile_log2"]) == [0, 0, 3, 4, 4]
            # b's runs are half lines, continued by the next tile along another dim: such tiles
            # are started in pairs on one XCD
            assert plan["tile_group"] == 2, (c.name, plan["tile_group"])
        else:
            assert plan["lds_bytes"] == 16 * 1024
    # an extent that is not a multiple of its tile extent clips tiles: general form
    a = View.empty("float", (48, 100)).permute(1, 0)
    plan = ocn.plan_binary("add", fake(a, 0), fake(View.empty("float", (100, 48)), 1), fake(View.empty("float", (100, 48)), 2))
    assert plan["kernel"] == "ew_tiled" and not plan["unclipped"]
    # a flipped staged input has a negative stride inside the tile: general form
    f = View.empty("float", (64, 128)).permute(1, 0).flip(1)
    plan = ocn.plan_binary("add", fake(f, 0), fake(View.empty("float", (128, 64)), 1), fake(View.empty("float", (128, 64)), 2))
    assert plan["kernel"] == "ew_tiled" and not plan["unclipped"]


def test_full_reduction_plan_is_two_pass_and_flat():
    c = configs.config4(64, 64, 1 << 28)[3]
    plan = ocn.plan_reduce("sum", fake(c.inputs[0], 0), [0], fake(c.out, 2))
    assert plan["kernel"] == "red_rows" and plan["red_size"] == (1 << 28,) and plan["ndim"] == 0
    assert plan["passes"] == 2 and plan["split"] > 1 and plan["vec"] == 16
    assert plan["compute_dtype"] == "int64"


def test_axis_reduction_plans():
    c4 = configs.config4(16384, 4096, 1024)
    a, b = c4[0], c4[1]
    p1 = ocn.plan_reduce("sum", fake(a.inputs[0], 0), [1], fake(a.out, 2))
    assert p1["kernel"] == "red_rows" and p1["size"] == (16384,) and p1["red_size"] == (4096,) and p1["passes"] == 1
    p0 = ocn.plan_reduce("sum", fake(b.inputs[0], 0), [0], fake(b.out, 2))
    assert p0["kernel"] == "red_cols" and p0["size"] == (4096,) and p0["red_size"] == (16384,)
    assert p0["split"] > 1 and p0["passes"] == 2
    assert p0["compute_dtype"] == "double"
    # reducing two adjacent axes of a contiguous tensor merges them
    v = View.empty("float", (6, 10, 12, 8))
    out = View.empty("float", (6, 8))
    p = ocn.plan_reduce("sum", fake(v, 0), [1, 2], fake(out, 2))
    assert p["red_size"] == (120,) and p["size"] == (6, 8)


@pytest.mark.parametrize("seed", range(30))
def test_reduce_plan_preserves_addend_sets(seed):
    rng = rng_for(7500 + seed)
    shape = random_shape(rng, max_ndim=5, max_elems=500)
    if not shape or 0 in shape:
        return
    a = random_strided_view(rng, "float", shape, allow_broadcast=False)
    naxes = int(rng.integers(1, len(shape) + 1))
    axes = sorted(int(x) for x in rng.permutation(len(shape))[:naxes])
    kept = [s for d, s in enumerate(shape) if d not in axes]
    out = random_strided_view(rng, "float", kept, writable=True)
    plan = ocn.plan_reduce("sum", fake(a, 0), axes, fake(out, 2))
    # raw: map output offset -> sorted input offsets
    raw = {}
    for idx in itertools.product(*[range(s) for s in shape]):
        kidx = [i for d, i in enumerate(idx) if d not in axes]
        oo = out.offset + sum(i * s for i, s in zip(kidx, out.strides))
        ao = a.offset + sum(i * s for i, s in zip(idx, a.strides))
        raw.setdefault(oo, []).append(ao)
    got = {}
    for kidx in itertools.product(*[range(s) for s in plan["size"]]):
        oo = plan["offset_out"] + sum(i * s for i, s in zip(kidx, plan["stride_out"]))
        base = plan["offset_a"] + sum(i * s for i, s in zip(kidx, plan["stride_a"]))
        for ridx in itertools.product(*[range(s) for s in plan["red_size"]]):
            got.setdefault(oo, []).append(base + sum(i * s for i, s in zip(ridx, plan["red_stride_a"])))
    assert {k: sorted(v) for k, v in raw.items()} == {k: sorted(v) for k, v in got.items()}


def test_vector_length_gives_the_widest_operand_sixteen_bytes():
    # per lane and vector the widest operand moves one 16-byte piece and the others one narrower
    # piece each, but no operand less than 4 bytes where the output's 16-byte limit allows it
    def vec(din, dout):
        return ocn.plan_unary("ident", fake(View.empty(din, (1 << 16,)), 0), fake(View.empty(dout, (1 << 16,)), 2))["vec"]
    assert vec("int8", "int32") == 4 and vec("half", "float") == 4 and vec("float", "double") == 2
    assert vec("double", "int16") == 2 and vec("double", "float") == 2 and vec("cdouble", "bool") == 4
    assert vec("float", "float") == 4 and vec("int8", "int8") == 16 and vec("cdouble", "cdouble") == 1
    assert vec("double", "int8") == 4 and vec("float", "int8") == 4 and vec("int8", "double") == 2


def test_general_form_layout_and_short_fastest_axes():
    # channel-last -> channel-first copy: with 4 channels the all-vector tiled form applies;
    # with 3 it cannot (3 is not a multiple of any tile extent), and a 12-byte axis is not
    # worth staging: the input is read in place, along the output's order
    def nhwc_to_nchw(c):
        a = View.empty("float", (8, 64, 64, c)).permute(0, 3, 1, 2)
        return ocn.plan_unary("ident", fake(a, 0), fake(View.empty("float", (8, c, 64, 64)), 2))
    p4, p3 = nhwc_to_nchw(4), nhwc_to_nchw(3)
    assert p4["kernel"] == "ew_tiled" and p4["unclipped"] and p4["stage_a"]
    assert p3["kernel"] == "ew_generic" and not p3["stage_a"] and p3["vec"] == 4
    # a transpose with odd extents: general form, with the larger tiles it prefers
    a = View.empty("float", (701, 500)).permute(1, 0)
    p = ocn.plan_binary("add", fake(a, 0), fake(View.empty("float", (500, 701)), 1), fake(View.empty("float", (500, 701)), 2))
    assert p["kernel"] == "ew_tiled" and not p["unclipped"] and p["tile_log2"] == (6, 6)


def test_reduction_layouts():
    def plan(a, axes, odt="double"):
        kept = [s for d, s in enumerate(a.sizes) if d not in axes]
        return ocn.plan_reduce("sum", fake(a, 0), list(axes), fake(View.empty(odt, kept), 2))
    # rows of any length, long or short, share lanes; a full reduction of a strided view is
    # split over workgroups like a contiguous one
    assert plan(View.empty("float", (1000, 7)), [1])["kernel"] == "red_rows"
    assert plan(View.empty("float", (1000, 64)), [1])["kernel"] == "red_rows"
    p = plan(View.empty("float", (1 << 22,)).slice(0, 0, 1 << 22, 2), [0])
    assert p["kernel"] == "red_rows" and p["passes"] == 2 and p["vec"] == 1
    # few columns: still the column kernel (several rows per wavefront)
    p = plan(View.empty("float", (1 << 20, 16)), [0])
    assert p["kernel"] == "red_cols" and p["passes"] == 2
    # no contiguous axis at all
    assert plan(View.empty("float", (300, 50, 2)).select(2, 1), [0])["kernel"] == "red_rows"
