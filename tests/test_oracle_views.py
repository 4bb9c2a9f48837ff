"""Invariants of the oracle under view manipulation (sections 3.1.3 and 4 of the paper:
strides give broadcasting, axis manipulation and views on regularly indexed subtensors)."""
import numpy as np
import pytest

from oracle import binding as O
from workloads.values import random_view, rng_for
from workloads.views import View, contiguous_strides


def test_transpose_twice_is_identity():
    rng = rng_for(61)
    a = random_view(rng, "float", (6, 7, 8))
    t = View.empty("float", (8, 6, 7))
    O.cast_copy(a.permute(2, 0, 1), t)               # materialise the permuted view
    back = View.empty("float", (6, 7, 8))
    O.cast_copy(t.permute(1, 2, 0), back)            # and permute back
    assert np.array_equal(back.storage, a.storage)
    assert np.array_equal(t.to_numpy().view(np.uint32), a.to_numpy().transpose(2, 0, 1).view(np.uint32))


def test_broadcast_equals_explicit_replication():
    rng = rng_for(62)
    a = random_view(rng, "int32", (5, 6, 7))
    row = random_view(rng, "float", (1, 6, 1))
    out1 = View.empty("float", (5, 6, 7))
    O.binary("mul", a, row, out1)
    rep = View.from_numpy(np.ascontiguousarray(np.broadcast_to(row.to_numpy(), (5, 6, 7))))
    out2 = View.empty("float", (5, 6, 7))
    O.binary("mul", a, rep, out2)
    assert np.array_equal(out1.storage, out2.storage)
    # zero strides written explicitly, and lower-rank operands, mean the same thing
    out3 = View.empty("float", (5, 6, 7))
    O.binary("mul", a, row.broadcast_to((5, 6, 7)), out3)
    out4 = View.empty("float", (5, 6, 7))
    O.binary("mul", a, row.select(0, 0), out4)       # shape (6, 1): padded on the left
    assert np.array_equal(out1.storage, out3.storage) and np.array_equal(out1.storage, out4.storage)


def test_size_one_dimension_ignores_its_stride():
    rng = rng_for(63)
    a = random_view(rng, "float", (4, 5))
    b = random_view(rng, "float", (1, 5))
    weird = View(b.storage, b.dtype, b.sizes, (123456, 4), b.offset)
    o1, o2 = View.empty("float", (4, 5)), View.empty("float", (4, 5))
    O.binary("add", a, b, o1)
    O.binary("add", a, weird, o2)
    assert np.array_equal(o1.storage, o2.storage)


def test_operation_on_flipped_view_is_flip_of_operation():
    rng = rng_for(64)
    a = random_view(rng, "double", (9, 4))
    b = random_view(rng, "double", (9, 4))
    o1, o2 = View.empty("double", (9, 4)), View.empty("double", (9, 4))
    O.binary("sub", a, b, o1)
    O.binary("sub", a.flip(0), b.flip(0), o2.flip(0))
    assert np.array_equal(o1.storage, o2.storage)


def test_views_share_storage_and_gaps_are_untouched():
    # write through a stepped, offset view: only the addressed elements change
    out_full = View.empty("int16", (6, 10), fill=0x5A)
    target = out_full.slice(1, 1, 10, 3).slice(0, 0, 6, 2)       # shape (3, 3)
    rng = rng_for(65)
    src = random_view(rng, "int16", (3, 3))
    before = out_full.to_numpy().copy()
    O.cast_copy(src, target)
    after = out_full.to_numpy()
    assert np.array_equal(after[0:6:2, 1:10:3], src.to_numpy())
    mask = np.ones((6, 10), dtype=bool)
    mask[0:6:2, 1:10:3] = False
    assert np.array_equal(after[mask], before[mask])


def test_padded_rows_and_offsets_in_bytes():
    # rows padded to a byte pitch that is not a multiple of the row length
    storage = np.arange(4 + 5 * 28, dtype=np.uint8)
    v = View(storage, "int32", (5, 6), (28, 4), 4)                # 24 data bytes + 4 pad per row
    out = View.empty("int32", (5, 6))
    O.cast_copy(v, out)
    want = np.stack([storage[4 + r * 28: 4 + r * 28 + 24].view(np.int32) for r in range(5)])
    assert np.array_equal(out.to_numpy(), want)


def test_eight_dimensions():
    rng = rng_for(66)
    a = random_view(rng, "uint8", (2,) * 8)
    perm = (7, 3, 5, 1, 0, 6, 2, 4)
    out = View.empty("uint8", (2,) * 8)
    O.cast_copy(a.permute(*perm), out)
    assert np.array_equal(out.to_numpy(), a.to_numpy().transpose(perm))


def test_column_major_and_row_major_describe_the_same_operation():
    rng = rng_for(67)
    a = random_view(rng, "float", (5, 7))
    c_out = View.empty("float", (5, 7), order="C")
    f_out = View.empty("float", (5, 7), order="F")
    O.unary("neg", a, c_out)
    O.unary("neg", a, f_out)
    assert np.array_equal(c_out.to_numpy(), f_out.to_numpy())
    assert f_out.strides == contiguous_strides((5, 7), 4, "F") == (4, 20)


def test_scalar_operand_and_zero_sized_output():
    rng = rng_for(68)
    a = random_view(rng, "float", (3, 4))
    s = View.from_numpy(np.array(2.5, dtype=np.float32))           # ndim 0
    out = View.empty("float", (3, 4))
    O.binary("mul", a, s, out)
    assert np.array_equal(out.to_numpy(), a.to_numpy() * np.float32(2.5))
    z = View.empty("float", (0, 4))
    O.binary("mul", z, s, View.empty("float", (0, 4)))             # a no-op, not an error
