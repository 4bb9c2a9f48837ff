"""Every error the boundary documents is detected on the host, before anything is launched, so
these run without a GPU (fake device addresses are never dereferenced)."""
import ctypes as C

import numpy as np
import pytest

import paper_1810_08723_amd as ocn
from paper_1810_08723_amd import binding as B
from workloads.views import View

E = B.ERR


def T(dtype, sizes, strides=None, offset=0, base=0x1000000000, device=0):
    es = ocn.dtype_size(dtype)
    if strides is None:
        strides, acc = [], es
        for s in reversed(sizes):
            strides.insert(0, acc)
            acc *= max(s, 1)
    return ocn.Tensor(base, dtype, tuple(sizes), tuple(strides), offset, device)


def code(fn, *args, **kw):
    with pytest.raises(ocn.OcnError) as e:
        fn(*args, **kw)
    return e.value.code


A, Bb, O_ = 0x1000000000, 0x2000000000, 0x3000000000


def test_null_pointers():
    lib = B.lib()
    t = T("float", (4,)).desc()
    assert lib.ocn_binary(0, None, C.byref(t), C.byref(t), 0, None) == E["NULLPTR"]
    assert lib.ocn_unary(0, C.byref(t), None, 0, None) == E["NULLPTR"]
    assert lib.ocn_reduce(0, C.byref(t), None, 1, C.byref(t), None, 0, None) == E["NULLPTR"]
    assert lib.ocn_plan_unary(0, C.byref(t), C.byref(t), 0, None) == E["NULLPTR"]
    assert code(ocn.plan_binary, "add", T("float", (4,), base=0), T("float", (4,), base=Bb), T("float", (4,), base=O_)) == E["NULLPTR"]


def test_bad_dtype_op_ndim_shape():
    a, b, o = T("float", (4, 5), base=A), T("float", (4, 5), base=Bb), T("float", (4, 5), base=O_)
    bad = ocn.Tensor(A, 17, (4, 5), (20, 4))
    assert code(ocn.plan_binary, "add", bad, b, o) == E["DTYPE"]
    lib = B.lib()
    info = B.OcnPlanInfo()
    assert lib.ocn_plan_binary(99, C.byref(a.desc()), C.byref(b.desc()), C.byref(o.desc()), 0, C.byref(info)) == E["OP"]
    nine = a.desc()
    nine.ndim = 9
    assert lib.ocn_plan_binary(0, C.byref(nine), C.byref(b.desc()), C.byref(o.desc()), 0, C.byref(info)) == E["NDIM"]
    eight = T("uint8", (2,) * 8, base=A)
    assert ocn.plan_unary("ident", eight, T("uint8", (2,) * 8, base=O_))["kernel"] == "ew_rows"  # 8 dims are fine
    assert code(ocn.plan_binary, "add", T("float", (5, 4), base=A), b, o) == E["SHAPE"]
    assert code(ocn.plan_binary, "add", T("float", (2, 4, 5), base=A), b, o) == E["SHAPE"]      # rank above out's
    assert code(ocn.plan_binary, "add", T("float", (-1, 5), base=A), b, o) == E["SHAPE"]


def test_operation_not_defined_for_type():
    f = lambda dt, base: T(dt, (4,), base=base)
    assert code(ocn.plan_binary, "band", f("float", A), f("float", Bb), f("float", O_)) == E["DTYPE"]
    assert code(ocn.plan_binary, "lt", f("cfloat", A), f("cfloat", Bb), f("bool", O_)) == E["DTYPE"]
    assert code(ocn.plan_binary, "max", f("cfloat", A), f("cfloat", Bb), f("cfloat", O_)) == E["DTYPE"]
    assert code(ocn.plan_binary, "add", f("bool", A), f("bool", Bb), f("bool", O_)) == E["DTYPE"]
    assert code(ocn.plan_unary, "abs", f("bool", A), f("bool", O_)) == E["DTYPE"]
    assert code(ocn.plan_unary, "bnot", f("cdouble", A), f("cdouble", O_)) == E["DTYPE"]
    # the modulus of a complex tensor is defined: computed in the input's type, a real result
    p = ocn.plan_unary("abs", f("cdouble", A), f("double", O_))
    assert p["compute_dtype"] == "cdouble" and p["specialised"]
    assert ocn.plan_unary("abs", f("cfloat", A), f("double", O_))["compute_dtype"] == "cfloat"
    ocn.plan_unary("abs", f("cfloat", A), f("float", O_), ocn.STRICT_TYPES)      # accepted
    assert code(ocn.plan_unary, "abs", f("cfloat", A), f("double", O_), ocn.STRICT_TYPES) == E["DTYPE"]
    assert code(ocn.plan_unary, "sqrt", f("int32", A), f("int32", O_)) == E["DTYPE"]
    assert code(ocn.plan_reduce, "max", f("cfloat", A), [0], T("cfloat", (), base=O_)) == E["DTYPE"]


def test_strict_types_flag():
    a, b, o = T("int32", (4,), base=A), T("float", (4,), base=Bb), T("float", (4,), base=O_)
    assert ocn.plan_binary("mul", a, b, o)["kernel"] == "ew_rows"
    assert code(ocn.plan_binary, "mul", a, b, o, ocn.STRICT_TYPES) == E["DTYPE"]
    assert code(ocn.plan_binary, "mul", b, b, T("double", (4,), base=O_), ocn.STRICT_TYPES) == E["DTYPE"]
    assert ocn.plan_binary("mul", b, b, o, ocn.STRICT_TYPES)["kernel"] == "ew_rows"
    assert ocn.plan_binary("lt", b, b, T("bool", (4,), base=O_), ocn.STRICT_TYPES)["compute_dtype"] == "float"
    assert code(ocn.plan_unary, "ident", a, o, ocn.STRICT_TYPES) == E["DTYPE"]


def test_binary_compute_type_follows_the_operands_unless_the_destination_is_one_of_them():
    """The planner's compute type against the rule of section 3.2.1, for every triple of types:
    the destination's type when it is an operand's or holds the promoted type, else the
    promoted type; kernels specialised by type only ever run in the destination's type."""
    import exactmath as X
    for da in X.ALL:
        for db in X.ALL:
            for do in X.ALL:
                want = X.compute_type("add", da, db, do)
                if not X.binary_supported("add", want):
                    assert code(ocn.plan_binary, "add", T(da, (4,), base=A), T(db, (4,), base=Bb), T(do, (4,), base=O_)) == E["DTYPE"]
                    continue
                p = ocn.plan_binary("add", T(da, (4,), base=A), T(db, (4,), base=Bb), T(do, (4,), base=O_))
                assert p["compute_dtype"] == want, (da, db, do)
                assert not p["specialised"] or want == do
    f = lambda dt, base: T(dt, (4,), base=base)
    assert ocn.plan_binary("add", f("int32", A), f("int32", Bb), f("int8", O_))["compute_dtype"] == "int32"
    assert ocn.plan_binary("add", f("int8", A), f("int32", Bb), f("int8", O_))["compute_dtype"] == "int8"
    assert ocn.plan_binary("add", f("int8", A), f("uint8", Bb), f("int64", O_))["compute_dtype"] == "int64"
    assert ocn.plan_binary("add", f("double", A), f("double", Bb), f("float", O_))["compute_dtype"] == "double"
    # a bitwise operation on floating operands stays undefined whatever the destination
    assert code(ocn.plan_binary, "bxor", f("float", A), f("double", Bb), f("int32", O_)) == E["DTYPE"]


def test_device_mismatch():
    a, b = T("float", (4,), base=A, device=0), T("float", (4,), base=Bb, device=1)
    assert code(ocn.plan_binary, "add", a, b, T("float", (4,), base=O_)) == E["DEVICE"]
    assert code(ocn.plan_reduce, "sum", a, [0], T("float", (), base=O_, device=1)) == E["DEVICE"]


def test_alignment():
    assert code(ocn.plan_unary, "neg", T("float", (4,), offset=2, base=A), T("float", (4,), base=O_)) == E["ALIGN"]
    assert code(ocn.plan_unary, "neg", T("float", (4, 4), strides=(18, 4), base=A), T("float", (4, 4), base=O_)) == E["ALIGN"]
    assert code(ocn.plan_unary, "neg", T("float", (4,), base=A + 1), T("float", (4,), base=O_)) == E["ALIGN"]
    # complex types align to their real component
    assert ocn.plan_unary("conj", T("cdouble", (4,), offset=8, base=A), T("cdouble", (4,), base=O_))["kernel"] != "none"
    # a stride on a size-1 dim is never used, so it need not be aligned
    assert ocn.plan_unary("neg", T("float", (1, 4), strides=(3, 4), base=A), T("float", (1, 4), base=O_))["kernel"] == "ew_rows"


def test_output_must_not_overlap_itself():
    a = T("float", (4, 4), base=A)
    assert code(ocn.plan_unary, "neg", a, T("float", (4, 4), strides=(0, 4), base=O_)) == E["OVERLAP_OUT"]
    assert code(ocn.plan_unary, "neg", a, T("float", (4, 4), strides=(8, 4), base=O_)) == E["OVERLAP_OUT"]
    assert code(ocn.plan_unary, "neg", a, T("float", (4, 4), strides=(4, 4), base=O_)) == E["OVERLAP_OUT"]
    assert code(ocn.plan_reduce, "sum", a, [1], T("float", (4,), strides=(0,), base=O_)) == E["OVERLAP_OUT"]
    # interleaved but disjoint is fine
    assert ocn.plan_unary("neg", a, T("float", (4, 4), strides=(4, 16), base=O_))["kernel"] != "none"


def test_input_output_aliasing():
    a = T("float", (4, 4), base=A)
    same = T("float", (4, 4), base=A)
    assert ocn.plan_unary("neg", a, same)["kernel"] == "ew_rows"                     # in place: the identical view
    assert ocn.plan_binary("add", a, T("float", (4, 4), base=Bb), same)["kernel"] == "ew_rows"
    shifted = T("float", (4, 4), offset=4, base=A)
    assert code(ocn.plan_unary, "neg", a, shifted) == E["ALIAS"]                     # overlapping, not identical
    transposed = T("float", (4, 4), strides=(4, 16), base=A)
    assert code(ocn.plan_unary, "neg", a, transposed) == E["ALIAS"]                  # in-place transpose
    other_type = T("int32", (4, 4), base=A)
    assert ocn.plan_unary("ident", a, other_type)["kernel"] == "ew_rows"             # same view, same element size
    narrower = T("int16", (4, 4), base=A)
    assert code(ocn.plan_unary, "ident", a, narrower) == E["ALIAS"]
    assert code(ocn.plan_reduce, "sum", a, [1], T("float", (4,), base=A)) == E["ALIAS"]
    disjoint = T("float", (4, 4), offset=64, base=A)
    assert ocn.plan_unary("neg", a, disjoint)["kernel"] == "ew_rows"


def test_reduce_arguments():
    a = T("float", (4, 6), base=A)
    assert code(ocn.plan_reduce, "sum", a, [2], T("float", (4,), base=O_)) == E["SHAPE"]
    assert code(ocn.plan_reduce, "sum", a, [1, 1], T("float", (), base=O_)) == E["SHAPE"]
    assert code(ocn.plan_reduce, "sum", a, [1], T("float", (6,), base=O_)) == E["SHAPE"]
    assert code(ocn.plan_reduce, "sum", a, [1], T("float", (4, 1), base=O_)) == E["SHAPE"]
    e = T("float", (4, 0), base=A)
    assert code(ocn.plan_reduce, "max", e, [1], T("float", (4,), base=O_)) == E["EMPTY"]
    assert ocn.plan_reduce("sum", e, [1], T("float", (4,), base=O_))["kernel"] == "red_generic"
    assert ocn.plan_reduce("max", e, [0], T("float", (0,), base=O_))["kernel"] == "none"


def test_workspace_errors_are_reported_before_any_launch():
    n = 1 << 24
    a = T("int8", (n,), base=A)
    out = T("int64", (), base=O_)
    need = ocn.reduce_workspace_bytes("sum", a, [0], out)
    assert need > 0 and need % 8 == 0
    lib = B.lib()
    ax = (C.c_int32 * 1)(0)
    rc = lib.ocn_reduce(0, C.byref(a.desc()), ax, 1, C.byref(out.desc()), None, 0, None)
    assert rc == E["WORKSPACE"]
    rc = lib.ocn_reduce(0, C.byref(a.desc()), ax, 1, C.byref(out.desc()), C.c_void_p(0x4000000000), need - 1, None)
    assert rc == E["WORKSPACE"]
    rc = lib.ocn_reduce(0, C.byref(a.desc()), ax, 1, C.byref(out.desc()), C.c_void_p(0x4000000010), need, None)
    assert rc == E["ALIGN"]
    assert ocn.reduce_workspace_bytes("sum", T("float", (64, 64), base=A), [1], T("float", (64,), base=O_)) == 0
    assert ocn.reduce_workspace_bytes("sum", a, [3], out) == 0          # invalid arguments: 0, the call reports why


def test_zero_sized_output_is_a_noop_even_with_null_storage():
    z = ocn.Tensor(0, "float", (0, 4), (16, 4))
    assert ocn.plan_binary("add", z, z, z)["kernel"] == "none"
    lib = B.lib()
    assert lib.ocn_binary(0, C.byref(z.desc()), C.byref(z.desc()), C.byref(z.desc()), 0, None) == 0
