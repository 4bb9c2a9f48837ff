"""Pins for tensors stored in the other byte order (section 3.1.3 of the paper: operations can
be applied in either byte order).  The oracle un-reverses each scalar on load and reverses it on
store; pinned against hand-written big-endian bytes, against numpy's byteswap (a library
routine with the same definition) and by the invariant that the byte order of an operand never
changes a value."""
import numpy as np
import pytest

from oracle import binding as O

from workloads.values import random_view, rng_for
from workloads.views import DTYPE_NAMES, View, itemsize


def _flagged(raw: bytes, dtype, sizes):
    """A contiguous view over hand-written bytes, declared to be in the other byte order."""
    es = itemsize(dtype)
    strides, acc = [], es
    for n in reversed(sizes):
        strides.insert(0, acc)
        acc *= n
    return View(np.frombuffer(raw, dtype=np.uint8).copy(), dtype, tuple(sizes), tuple(strides), 0, True)


def test_hand_written_big_endian_values():
    # int32 1, -2 and float 1.0, -2.5 as a big-endian machine stores them
    v = _flagged(bytes([0, 0, 0, 1, 0xFF, 0xFF, 0xFF, 0xFE]), "int32", (2,))
    out = View.empty("int64", (2,))
    O.cast_copy(v, out)
    assert out.to_numpy().tolist() == [1, -2]
    v = _flagged(bytes([0x3F, 0x80, 0, 0, 0xC0, 0x20, 0, 0]), "float", (2,))
    out = View.empty("double", (2,))
    O.cast_copy(v, out)
    assert out.to_numpy().tolist() == [1.0, -2.5]
    # a complex element is two scalars, each reversed on its own: (1 + 2i) in single precision
    v = _flagged(bytes([0x3F, 0x80, 0, 0, 0x40, 0, 0, 0]), "cfloat", (1,))
    out = View.empty("cdouble", (1,))
    O.cast_copy(v, out)
    assert out.to_numpy()[0] == 1 + 2j
    # half 1.5 = 0x3E00, uint16 258 = 0x0102, one byte types are unaffected
    v = _flagged(bytes([0x3E, 0x00]), "half", (1,))
    out = View.empty("float", (1,))
    O.cast_copy(v, out)
    assert out.to_numpy()[0] == 1.5
    v = _flagged(bytes([0x01, 0x02]), "uint16", (1,))
    out = View.empty("int32", (1,))
    O.cast_copy(v, out)
    assert out.to_numpy()[0] == 258
    v = _flagged(bytes([0x85]), "int8", (1,))
    O.cast_copy(v, out)
    assert out.to_numpy()[0] == -123
    # storing: the value 258 into a flagged uint16 output leaves bytes 01 02
    src = View.from_numpy(np.array([258, 1], dtype=np.int32))
    dst = View(np.zeros(4, dtype=np.uint8), "uint16", (2,), (2,), 0, True)
    O.cast_copy(src, dst)
    assert dst.storage.tolist() == [1, 2, 0, 1]


@pytest.mark.parametrize("dtype", DTYPE_NAMES)
def test_view_helper_matches_numpy_byteswap(dtype):
    rng = rng_for(17000)
    a = random_view(rng, dtype, (5, 7))
    b = a.in_other_byte_order()
    assert b.byteswapped and np.array_equal(a.to_numpy().view(np.uint8), b.to_numpy().view(np.uint8))
    if dtype != "chalf":
        arr = a.to_numpy()
        c = View.from_numpy(arr).in_other_byte_order()
        assert np.array_equal(c.storage, arr.byteswap().reshape(-1).view(np.uint8))


@pytest.mark.parametrize("dtype", DTYPE_NAMES)
def test_byte_order_of_an_operand_never_changes_a_value(dtype):
    rng = rng_for(17001)
    a = random_view(rng, dtype, (6, 9)).permute(1, 0)
    b = random_view(rng, dtype, (9, 6))
    af, bf = a.in_other_byte_order(), b.in_other_byte_order()
    op = "land" if dtype == "bool" else "add"
    want = View.empty(dtype, (9, 6))
    O.binary(op, a, b, want)
    for x, y in ((af, b), (a, bf), (af, bf)):
        got = View.empty(dtype, (9, 6))
        O.binary(op, x, y, got)
        assert np.array_equal(got.storage, want.storage)
    # a flagged output holds the same values with every scalar reversed
    got = View(np.full(want.storage.size, 0xA5, dtype=np.uint8), dtype, (9, 6), want.strides, 0, True)
    O.binary(op, af, b, got)
    assert np.array_equal(got.storage, want.in_other_byte_order().storage)
    assert np.array_equal(got.to_numpy().view(np.uint8), want.to_numpy().view(np.uint8))
    # casts and reductions read flagged inputs the same way
    wide = {"bool": "int32", "chalf": "cdouble", "cfloat": "cdouble", "cdouble": "cdouble"}.get(dtype, "double")
    w1, w2 = View.empty(wide, (9, 6)), View.empty(wide, (9, 6))
    O.cast_copy(a, w1)
    O.cast_copy(af, w2)
    assert np.array_equal(w1.storage, w2.storage)
    r1, r2 = View.empty(wide, (9,)), View.empty(wide, (9,))
    O.reduce("sum", a, [1], r1)
    O.reduce("sum", af, [1], r2)
    assert np.array_equal(r1.storage, r2.storage)
    r3 = View(np.zeros(r1.storage.size, dtype=np.uint8), wide, (9,), r1.strides, 0, True)
    O.reduce("sum", af, [1], r3)
    assert np.array_equal(r3.storage, r1.in_other_byte_order().storage)
