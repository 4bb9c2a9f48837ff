"""Pins for the oracle's index binding, gather and scatter: NumPy's own fancy and boolean
indexing on materialised arrays (the library routines these operations reduce to), counts,
ordering, and round trips."""
import numpy as np
import pytest

from oracle import indexing as OI
from workloads.values import random_view, rng_for
from workloads.views import View


def test_index_binding_wraps_negative_and_flags_invalid():
    idx = np.array([[0, 3, -1], [-4, 4, -5]], dtype=np.int64)
    offs, bad = OI.index_offsets(idx, 4, 24)
    assert bad == 2
    assert offs.tolist() == [[0, 72, 72], [0, 0, 0]]          # 4 and -5 are outside [-4, 4)
    rng = rng_for(8200)
    idx = rng.integers(-50, 50, size=200)
    offs, bad = OI.index_offsets(idx, 50, 8)
    assert bad == 0 and np.array_equal(offs, (idx % 50) * 8)   # Python's modulo is the wrap for valid indices


def test_mask_offsets_follow_numpy_nonzero_order():
    rng = rng_for(8201)
    m = rng.random((5, 7, 3)) < 0.4
    mask = View.from_numpy(m).permute(2, 0, 1)               # a strided mask: shape (3, 5, 7)
    logical = mask.to_numpy()
    strides = (8, 1000, 24)                                    # arbitrary target strides
    offs = OI.mask_offsets(mask, strides)
    nz = np.argwhere(logical)                                  # row-major order of selected positions
    assert len(offs) == int(logical.sum())
    assert np.array_equal(offs, (nz * np.array(strides)).sum(axis=1))


def test_gather_equals_numpy_boolean_and_fancy_indexing():
    rng = rng_for(8202)
    a = random_view(rng, "float", (9, 6, 4), specials=False)
    arr = a.to_numpy()
    # element-wise mask over the whole tensor
    m = rng.random((9, 6, 4)) < 0.3
    offs = OI.mask_offsets(View.from_numpy(m), a.strides)
    out = View.empty("float", (len(offs),))
    OI.gather(View(a.storage, "float", (), (), a.offset), offs, out, 0, a.storage.size - 4)
    assert np.array_equal(out.to_numpy(), arr[m])
    # index array along axis 0 selects whole [6, 4] slabs, negative indices included
    idx = np.array([8, -1, 0, 3, 3, -9], dtype=np.int64)
    offs, bad = OI.index_offsets(idx, 9, a.strides[0])
    assert bad == 0
    out = View.empty("float", (6, 6, 4))
    inner = View(a.storage, "float", (6, 4), a.strides[1:], a.offset)
    OI.gather(inner, offs, out, 0, 8 * a.strides[0])
    assert np.array_equal(out.to_numpy(), arr[idx])
    # index array along the last axis of a permuted view
    p = a.permute(2, 0, 1)                                      # shape (4, 9, 6)
    idx = np.array([5, 0, -2], dtype=np.int64)
    offs, _ = OI.index_offsets(idx, 6, p.strides[2])
    out = View.empty("float", (3, 4, 9))
    OI.gather(View(p.storage, "float", (4, 9), p.strides[:2], p.offset), offs, out, 0, 5 * p.strides[2])
    assert np.array_equal(out.to_numpy(), np.moveaxis(p.to_numpy()[:, :, idx], 2, 0))


def test_scatter_equals_numpy_assignment_and_round_trip():
    rng = rng_for(8203)
    a = random_view(rng, "int32", (12, 5))
    before = a.to_numpy().copy()
    m = rng.random((12, 5)) < 0.5
    offs = OI.mask_offsets(View.from_numpy(m), a.strides)
    vals = random_view(rng, "int32", (len(offs),))
    OI.scatter(vals, offs, View(a.storage, "int32", (), (), a.offset), 0, a.storage.size - 4)
    want = before.copy()
    want[m] = vals.to_numpy()
    assert np.array_equal(a.to_numpy(), want)
    back = View.empty("int32", (len(offs),))
    OI.gather(View(a.storage, "int32", (), (), a.offset), offs, back, 0, a.storage.size - 4)
    assert np.array_equal(back.to_numpy(), vals.to_numpy())


def test_out_of_range_offsets_are_skipped():
    a = View.from_numpy(np.arange(10, dtype=np.int16))
    out = View.empty("int16", (4,))
    before = out.storage.copy()
    OI.gather(View(a.storage, "int16", (), (), 0), np.array([0, 40, -2, 18], dtype=np.int64), out, 0, 18)
    got = out.to_numpy()
    assert got[0] == 0 and got[3] == 9
    assert np.array_equal(out.storage[2:6], before[2:6])      # rows 1 and 2 untouched


def test_gather_and_scatter_between_byte_orders_move_values():
    """Section 3.1.3: a tensor may hold its data in the other byte order.  Indexed copies move
    values: bytes written by hand in big-endian order come out as the native numbers, complex
    elements part by part, and a scatter into such a tensor writes big-endian bytes."""
    be = np.array([1, 258, -2, 0x01020304], dtype=">i4")            # 00 00 00 01 | 00 00 01 02 | ff ff ff fe | 01 02 03 04
    src = View(np.frombuffer(be.tobytes(), dtype=np.uint8).copy(), "int32", (), (), 0, True)
    assert list(src.storage[:8]) == [0, 0, 0, 1, 0, 0, 1, 2]
    out = View.empty("int32", (3,))
    OI.gather(src, np.array([12, 0, 8], dtype=np.int64), out, 0, 12)
    assert list(out.to_numpy()) == [0x01020304, 1, -2]
    # the same order on both sides: bytes are copied as they are
    same = View(np.zeros(12, dtype=np.uint8), "int32", (3,), (4,), 0, True)
    OI.gather(src, np.array([4, 4, 0], dtype=np.int64), same, 0, 12)
    assert list(same.storage) == [0, 0, 1, 2, 0, 0, 1, 2, 0, 0, 0, 1]
    assert list(same.to_numpy()) == [258, 258, 1]
    # complex: each part is a scalar of its own
    z = np.array([1.5 - 2.25j, 3.0 + 0.5j], dtype=np.complex64)
    zb = z.view(np.float32).astype(">f4").tobytes()
    zsrc = View(np.frombuffer(zb, dtype=np.uint8).copy(), "cfloat", (), (), 0, True)
    zout = View.empty("cfloat", (2,))
    OI.gather(zsrc, np.array([8, 0], dtype=np.int64), zout, 0, 8)
    assert list(zout.to_numpy()) == [z[1], z[0]]
    # scatter native values into a big-endian tensor
    vals = View.from_numpy(np.array([7, -1], dtype=np.int16))
    tgt = View(np.zeros(8, dtype=np.uint8), "int16", (), (), 0, True)
    OI.scatter(vals, np.array([6, 2], dtype=np.int64), tgt, 0, 6)
    assert list(tgt.storage) == [0, 0, 0xff, 0xff, 0, 0, 0, 7]
    # round trip through the other order gives the data back
    rng = rng_for(16100)
    a = random_view(rng, "double", (40,))
    swapped = View.empty("double", (40,))
    swapped = View(swapped.storage, "double", (40,), (8,), 0, True)
    offs = (rng.permutation(40) * 8).astype(np.int64)
    OI.gather(View(a.storage, "double", (), (), 0), offs, swapped, 0, 39 * 8)
    back = View.empty("double", (40,))
    OI.scatter(swapped, offs, View(back.storage, "double", (), (), 0), 0, 39 * 8)
    assert np.array_equal(back.storage, a.storage)
    assert np.array_equal(swapped.to_numpy().view(np.uint64), a.to_numpy()[offs // 8].view(np.uint64))
