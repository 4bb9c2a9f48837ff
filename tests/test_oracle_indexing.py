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
