"""GPU parity of every unary and binary operation on every compute type, plus mixed-type calls
that go through the generic-dtype kernel.  Bit-exact against the oracle."""
import numpy as np
import pytest

import exactmath as X
import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu

LAYOUTS = ("rows", "tiled", "strided")


def _operands(rng, da, db, dout, layout):
    if layout == "rows":
        a = random_view(rng, da, (33, 150))
        b = random_view(rng, db, (1, 150))                       # broadcast row
        return a, b, View.empty(dout, (33, 150))
    if layout == "tiled":
        a = random_view(rng, da, (40, 66))
        b = random_view(rng, db, (66, 40)).permute(1, 0)         # transposed operand
        return a, b, View.empty(dout, (40, 66))
    a = random_view(rng, da, (12, 9, 14)).slice(2, 0, 14, 2)     # stepped
    b = random_view(rng, db, (12, 9, 7)).flip(1)
    return a, b, View.empty(dout, (12, 9, 7), order="F")


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("T", X.ALL)
def test_homogeneous_binary_ops(T, layout):
    rng = rng_for(9000 + 17 * X.ALL.index(T) + LAYOUTS.index(layout))
    for op in X.ARITH + X.BITWISE:
        if not X.binary_supported(op, T):
            continue
        print("binary", op, T, layout, flush=True)
        a, b, out = _operands(rng, T, T, T, layout)
        H.check_binary(op, a, b, out)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("T", X.ALL)
def test_comparisons_and_logical(T, layout):
    rng = rng_for(9200 + 17 * X.ALL.index(T) + LAYOUTS.index(layout))
    for op in X.COMPARE + X.LOGICAL:
        if not X.binary_supported(op, X.compute_type(op, T, T, "bool")):
            continue
        print("predicate", op, T, layout, flush=True)
        a, b, out = _operands(rng, T, T, "bool", layout)
        b.storage[: b.storage.size // 2] = a.storage[: b.storage.size // 2]   # plenty of equal pairs
        H.check_binary(op, a, b, out)


@pytest.mark.parametrize("T", X.ALL)
def test_unary_ops(T):
    rng = rng_for(9400 + X.ALL.index(T))
    for op in X.UNARY:
        if not X.unary_supported(op, "bool" if op == "lnot" else T):
            continue
        for layout in ("rows", "tiled"):
            print("unary", op, T, layout, flush=True)
            if layout == "rows":
                a, out = random_view(rng, T, (29, 77)), View.empty(T, (29, 77))
            else:
                a, out = random_view(rng, T, (77, 29)).permute(1, 0), View.empty(T, (29, 77))
            H.check_unary(op, a, out)


MIXED = [("add", "int32", "float", "float"), ("sub", "double", "int8", "int16"), ("mul", "half", "uint8", "half"),
         ("div", "int64", "double", "float"), ("mul", "cfloat", "half", "chalf"), ("max", "bool", "int16", "double"),
         ("add", "uint64", "int64", "double"), ("mul", "float", "cdouble", "cfloat"), ("bxor", "uint8", "int64", "int32"),
         ("lt", "int8", "uint8", "bool"), ("ge", "int64", "float", "bool"), ("eq", "cfloat", "cdouble", "bool"),
         ("absgt", "chalf", "int32", "bool"), ("ne", "uint64", "int64", "uint8"), ("land", "float", "int8", "bool"),
         ("lor", "cdouble", "bool", "float"), ("le", "half", "int16", "int64"), ("absgt", "int8", "uint64", "bool"),
         # destinations that are neither an operand's type nor hold the promoted type: the operation
         # runs in the promoted type, the result is converted on store
         ("add", "int32", "int32", "int8"), ("mul", "int32", "int32", "int8"), ("add", "double", "double", "float"),
         ("sub", "int16", "uint8", "int8"), ("div", "float", "int32", "half"), ("mul", "uint64", "int8", "uint16"),
         ("mul", "cdouble", "float", "cfloat"), ("add", "half", "half", "int16"), ("mul", "chalf", "half", "half"),
         ("sub", "half", "uint8", "int32"), ("bxor", "int32", "uint8", "int8"), ("band", "uint16", "bool", "uint8"),
         ("min", "int64", "int64", "int16"), ("max", "float", "float", "half")]


@pytest.mark.parametrize("op,da,db,dout", MIXED)
def test_mixed_types_through_the_generic_kernel(op, da, db, dout):
    rng = rng_for(9600 + sum(map(ord, op + da + db + dout)))
    for layout in LAYOUTS:
        a, b, out = _operands(rng, da, db, dout, layout)
        H.check_binary(op, a, b, out)


CONVERT_ON_LOAD = [("int32", "float", "float"), ("float", "int32", "float"), ("half", "float", "float"),
                   ("float", "half", "float"), ("float", "double", "double"), ("double", "float", "double"),
                   ("int32", "double", "double"), ("double", "int32", "double"), ("int64", "double", "double"),
                   ("double", "int64", "double"), ("float", "cfloat", "cfloat"), ("cfloat", "float", "cfloat"),
                   ("double", "cdouble", "cdouble"), ("cdouble", "double", "cdouble")]


@pytest.mark.parametrize("da,db,dout", CONVERT_ON_LOAD)
def test_mixed_types_with_kernels_that_convert_on_load(da, db, dout):
    import paper_1810_08723_amd as ocn
    rng = rng_for(9700 + sum(map(ord, da + db + dout)))
    for op in ("add", "sub", "mul", "div"):
        for layout in LAYOUTS + ("unclipped", "long rows"):
            if layout == "unclipped":          # power-of-two transpose: the all-vector tiled form
                a = random_view(rng, da, (64, 128))
                b = random_view(rng, db, (128, 64)).permute(1, 0)
                out = View.empty(dout, (64, 128))
            elif layout == "long rows":        # several vectors per lane and a ragged tail
                a = random_view(rng, da, (3, 5003))
                b = random_view(rng, db, (3, 5003))
                out = View.empty(dout, (3, 5003))
            else:
                a, b, out = _operands(rng, da, db, dout, layout)
            dv = H.DeviceViews()
            plan = ocn.plan_binary(op, dv.tensor(a), dv.tensor(b), dv.tensor(out))
            assert plan["specialised"], (op, da, db, dout, layout)
            print("mixed", op, da, db, dout, layout, plan["kernel"], flush=True)
            H.check_binary(op, a, b, out)


def test_lnot_and_casts_of_predicates_to_non_bool_outputs():
    rng = rng_for(9700)
    a = random_view(rng, "float", (50, 20))
    H.check_unary("lnot", a, View.empty("int32", (50, 20)))
    H.check_unary("lnot", a, View.empty("double", (50, 20)))
    H.check_binary("gt", a, random_view(rng, "float", (50, 20)), View.empty("half", (50, 20)))


def test_complex_multiply_is_not_contracted():
    # a fused multiply-add in (ac - bd) would change low bits; the oracle rounds all six operations
    rng = rng_for(9701)
    a = random_view(rng, "cfloat", (300, 64), specials=False)
    b = random_view(rng, "cfloat", (300, 64), specials=False)
    H.check_binary("mul", a, b, View.empty("cfloat", (300, 64)))
    H.check_binary("div", a, b, View.empty("cfloat", (300, 64)))
    ad = random_view(rng, "cdouble", (100, 64), specials=False)
    bd = random_view(rng, "cdouble", (100, 64), specials=False)
    H.check_binary("mul", ad, bd, View.empty("cdouble", (100, 64)))
    H.check_binary("div", ad, bd, View.empty("cdouble", (100, 64)))


def test_division_and_sqrt_are_correctly_rounded():
    rng = rng_for(9702)
    for dt in ("half", "float", "double"):
        a = random_view(rng, dt, (4000,))
        b = random_view(rng, dt, (4000,))
        H.check_binary("div", a, b, View.empty(dt, (4000,)))
        H.check_unary("sqrt", a, View.empty(dt, (4000,)))
    # denormal operands and results stay denormal (no flush to zero)
    tiny = View.from_numpy(np.array([1e-40, 3e-45, 1.1754944e-38, -2e-41] * 16, dtype=np.float32))
    H.check_binary("mul", tiny, View.from_numpy(np.full(64, 0.5, dtype=np.float32)), View.empty("float", (64,)))
    H.check_binary("add", tiny, tiny.fresh_copy(), View.empty("float", (64,)))
