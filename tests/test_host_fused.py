"""Host-side planning of the fused elementwise+reduce call: which kernel layout each kind of
operand pair gets, when the two-call fallback is planned, and the documented errors."""
import numpy as np
import pytest

import paper_1810_08723_amd as ocn
from workloads.views import View

E = ocn.binding.ERR


def fake(v, i):
    return ocn.Tensor(0x100000000 * (i + 1), v.dtype, v.sizes, v.strides, v.offset, 0)


def plan(ew, red, a, b, axes, out, mid):
    return ocn.plan_binary_reduce(ew, red, fake(a, 0), fake(b, 1), list(axes), fake(out, 2), mid)


def test_inner_product_along_the_fastest_axis_is_a_fused_rows_kernel():
    a, b = View.empty("float", (16384, 4096)), View.empty("float", (16384, 4096))
    p = plan("mul", "sum", a, b, (1,), View.empty("float", (16384,)), "float")
    assert p["fused"] and p["kernel"] == "red_rows" and p["passes"] == 1 and p["vec"] == 4
    assert p["size"] == (16384,) and p["red_size"] == (4096,) and p["compute_dtype"] == "double"
    # a full inner product of two flat vectors is split over the device and folded by a second launch
    x, y = View.empty("double", (1 << 24,)), View.empty("double", (1 << 24,))
    p = plan("mul", "sum", x, y, (0,), View.empty("double", ()), "double")
    assert p["fused"] and p["kernel"] == "red_rows" and p["split"] > 1 and p["passes"] == 2


def test_broadcast_row_and_column_operands():
    a = View.empty("float", (512, 1024))
    row = View.empty("float", (1024,))
    col = View.empty("float", (512, 1))
    # b is one row for every row of a: contiguous along the reduced axis, stride 0 across rows
    p = plan("sub", "sum", a, row, (1,), View.empty("float", (512,)), "float")
    assert p["fused"] and p["kernel"] == "red_rows"
    # b is one value per row: broadcast along the reduced (vectorised) axis
    p = plan("mul", "sum", a, col, (1,), View.empty("float", (512,)), "float")
    assert p["fused"] and p["kernel"] == "red_rows"
    # reducing over rows keeps the contiguous axis: the columns kernel
    p = plan("mul", "sum", a, row, (0,), View.empty("float", (1024,)), "float")
    assert p["fused"] and p["kernel"] == "red_cols"


def test_mismatched_layouts_use_the_generic_fused_kernel():
    a = View.empty("double", (64, 48))
    bt = View.empty("double", (48, 64)).permute(1, 0)
    p = plan("mul", "sum", a, bt, (1,), View.empty("double", (64,)), "double")
    assert p["fused"] and p["kernel"] == "red_generic"


def test_count_of_a_comparison_and_unfused_fallback():
    a, b = View.empty("cfloat", (1 << 20,)), View.empty("cfloat", (1 << 20,))
    p = plan("absgt", "sum", a, b, (0,), View.empty("int64", ()), "bool")
    assert p["fused"] and p["kernel"] == "red_rows" and p["compute_dtype"] == "int64"
    # no fused kernel for division or for mixed input types: planned as two calls
    f, g = View.empty("float", (1000, 100)), View.empty("float", (1000, 100))
    p = plan("div", "sum", f, g, (1,), View.empty("float", (1000,)), "float")
    assert not p["fused"] and p["passes"] >= 2
    i = View.empty("int32", (1000, 100))
    p = plan("mul", "sum", i, g, (1,), View.empty("float", (1000,)), "float")
    assert not p["fused"]
    t = fake(f, 0)
    need = ocn.binary_reduce_workspace_bytes("div", "sum", t, fake(g, 1), [1], fake(View.empty("float", (1000,)), 2), "float")
    assert need >= 1000 * 100 * 4


def test_errors():
    a, b = View.empty("float", (8, 6)), View.empty("float", (8, 6))
    out = View.empty("float", (8,))

    def code(*args):
        with pytest.raises(ocn.OcnError) as e:
            plan(*args)
        return e.value.code
    assert code("mul", "sum", a, View.empty("float", (8, 5)), (1,), out, "float") == E["SHAPE"]      # not broadcastable
    assert code("mul", "sum", a, b, (2,), out, "float") == E["SHAPE"]                                  # axis out of range
    assert code("mul", "sum", a, b, (1, 1), out, "float") == E["SHAPE"]                                # repeated axis
    assert code("mul", "sum", a, b, (1,), View.empty("float", (6,)), "float") == E["SHAPE"]            # wrong kept size
    assert code("band", "sum", a, b, (1,), out, "float") == E["DTYPE"]                                 # bitwise on floats
    assert code("mul", "max", View.empty("cfloat", (8, 6)), View.empty("cfloat", (8, 6)), (1,),
                View.empty("cfloat", (8,)), "cfloat") == E["DTYPE"]                                    # max of complex
    assert code("mul", "max", View.empty("float", (8, 0)), View.empty("float", (8, 0)), (1,), out, "float") == E["EMPTY"]
    with pytest.raises(ocn.OcnError) as e:   # output inside an input
        ocn.plan_binary_reduce("mul", "sum", fake(a, 0), fake(b, 1), [1],
                               ocn.Tensor(0x100000000, "float", (8,), (4,), 0, 0), "float")
    assert e.value.code == E["ALIAS"]
