"""GPU parity of index binding, mask compaction, gather and scatter against the oracle, bit for
bit (everything here is integer or byte work), plus end-to-end agreement with NumPy's fancy and
boolean indexing."""
import numpy as np
import pytest

import gpu_harness as H
from oracle import indexing as OI
from workloads.values import random_view, rng_for
from workloads.views import View, itemsize

pytestmark = pytest.mark.gpu


def _dev_i64(arr):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.int64)).to("cuda:0")


def _mask_offsets_gpu(mask: View, strides, capacity=None):
    import torch
    import paper_1810_08723_amd as ocn
    dv = H.DeviceViews()
    n = mask.numel
    cap = n if capacity is None else capacity
    offs = torch.full((max(cap, 0),), -7, dtype=torch.int64, device="cuda:0")
    count = torch.full((1,), -1, dtype=torch.int64, device="cuda:0")
    ocn.mask_offsets(dv.tensor(mask), list(strides), offs, count)
    torch.cuda.synchronize()
    return offs.cpu().numpy(), int(count.cpu()[0])


def test_index_binding():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17000)
    idx = rng.integers(-70, 70, size=(37, 53)).astype(np.int64)          # dim_size 64: some invalid
    iv = View.from_numpy(idx).permute(1, 0)                                # strided index tensor
    ov = View.empty("int64", (53, 37))
    dv = H.DeviceViews()
    bad = torch.full((1,), 123, dtype=torch.int64, device="cuda:0")
    ocn.index_offsets(dv.tensor(iv), 64, 24, dv.tensor(ov), bad)
    torch.cuda.synchronize()
    want, nbad = OI.index_offsets(iv.to_numpy(), 64, 24)
    got = View(dv.download(ov), "int64", ov.sizes, ov.strides, 0).to_numpy()
    assert np.array_equal(got, want) and int(bad.cpu()[0]) == nbad and nbad > 0
    # all valid; 1-D; zero-sized
    idx = rng.integers(-64, 64, size=(5000,)).astype(np.int64)
    ov = View.empty("int64", (5000,))
    dv = H.DeviceViews()
    ocn.index_offsets(dv.tensor(View.from_numpy(idx)), 64, -8, dv.tensor(ov), bad)
    torch.cuda.synchronize()
    want, nbad = OI.index_offsets(idx, 64, -8)
    assert np.array_equal(dv.download(ov).view(np.int64), want) and int(bad.cpu()[0]) == 0
    ocn.index_offsets(dv.tensor(View.empty("int64", (0,))), 64, 8, dv.tensor(View.empty("int64", (0,))), bad)
    torch.cuda.synchronize()
    assert int(bad.cpu()[0]) == 0


@pytest.mark.parametrize("shape", ((1,), (2,), (7,), (4096,), (100003,), (37, 53), (5, 1, 9, 11)))
def test_index_binding_contiguous_arrays(shape):
    """Contiguous index and offset arrays take the kernel with two indices per lane: odd counts,
    negative and invalid indices, and the capped grid (lanes loop)."""
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17010 + len(shape) + shape[0])
    idx = rng.integers(-70, 70, size=shape).astype(np.int64)               # dim_size 64: some invalid
    for cap in (None, 3):
        iv, ov = View.from_numpy(idx), View.empty("int64", shape)
        dv = H.DeviceViews()
        bad = torch.full((1,), 123, dtype=torch.int64, device="cuda:0")
        if cap:
            ocn.binding.set_max_launch_blocks(cap)
        try:
            ocn.index_offsets(dv.tensor(iv), 64, 24, dv.tensor(ov), bad)
            torch.cuda.synchronize()
        finally:
            if cap:
                ocn.binding.set_max_launch_blocks(0)
        want, nbad = OI.index_offsets(idx, 64, 24)
        got = View(dv.download(ov), "int64", ov.sizes, ov.strides, 0).to_numpy()
        assert np.array_equal(got, want) and int(bad.cpu()[0]) == nbad


@pytest.mark.parametrize("density", (0.0, 0.03, 0.5, 1.0))
def test_mask_offsets_contiguous(density):
    rng = rng_for(17100)
    n = 3 * 4096 * 5 + 1234                                               # several workgroups and a ragged tail
    m = rng.random(n) < density
    mask = View.from_numpy(m)
    got, count = _mask_offsets_gpu(mask, (4,))
    want = OI.mask_offsets(mask, (4,))
    assert count == len(want) == int(m.sum())
    assert np.array_equal(got[:count], want) and np.all(got[count:] == -7)
    # a 3-D contiguous mask bound to a permuted target: merged on the mask side only where both merge
    m3 = rng.random((33, 20, 50)) < density
    strides = (8, 8 * 33 * 50, 8 * 33)                                     # target stored as (1, 2, 0)
    got, count = _mask_offsets_gpu(View.from_numpy(m3), strides)
    want = OI.mask_offsets(View.from_numpy(m3), strides)
    assert count == len(want) and np.array_equal(got[:count], want)


def test_mask_offsets_strided_masks_capacity_and_degenerate():
    rng = rng_for(17101)
    m = rng.random((40, 33, 21)) < 0.4
    mask = View.from_numpy(m).permute(2, 0, 1).slice(1, 0, 40, 2)         # shape (21, 20, 33), strided
    strides = (4, 4 * 21 * 33, 4 * 21)
    got, count = _mask_offsets_gpu(mask, strides)
    want = OI.mask_offsets(mask, strides)
    assert count == len(want) and np.array_equal(got[:count], want)
    # capacity smaller than the count: the first `capacity` offsets, the full count
    got, count = _mask_offsets_gpu(mask, strides, capacity=100)
    assert count == len(want) and np.array_equal(got, want[:100])
    # unaligned contiguous mask (starts one byte into its storage), scalar mask, empty mask
    big = View.from_numpy(rng.random(10001) < 0.5)
    off1 = big.slice(0, 1, 10001, 1)
    got, count = _mask_offsets_gpu(off1, (2,))
    want = OI.mask_offsets(off1, (2,))
    assert count == len(want) and np.array_equal(got[:count], want)
    for val in (True, False):
        got, count = _mask_offsets_gpu(View.from_numpy(np.array(val)), ())
        assert count == int(val) and (not val or got[0] == 0)
    got, count = _mask_offsets_gpu(View.from_numpy(np.zeros((0, 5), dtype=np.bool_)), (40, 8), capacity=0)
    assert count == 0


def test_mask_offsets_large_by_properties():
    # more workgroup counts than one round of the scan holds (16384), and a ragged tail.  The
    # result is the only strictly increasing sequence of `count` selected positions, which is
    # checked as such; a window at the boundary between the rounds is compared with the oracle.
    rng = rng_for(17102)
    n = 16384 * 4096 + 3 * 4096 + 77
    m = rng.random(n, dtype=np.float32) < 0.02
    got, count = _mask_offsets_gpu(View.from_numpy(m), (8,), capacity=int(m.sum()) + 5)
    assert count == int(np.count_nonzero(m))
    sel = got[:count]
    assert np.all(sel % 8 == 0) and np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < 8 * n
    assert m[sel // 8].all() and np.all(got[count:] == -7)
    lo, hi = 16384 * 4096 - 3000, 16384 * 4096 + 3000
    want = OI.mask_offsets(View.from_numpy(m[lo:hi].copy()), (8,)) + 8 * lo
    first = int(np.count_nonzero(m[:lo]))
    assert np.array_equal(sel[first:first + len(want)], want)


@pytest.mark.parametrize("dt", ("int8", "half", "float", "double", "cfloat", "cdouble"))
def test_gather_scatter_elementwise_by_mask(dt):
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17200 + itemsize(dt))
    a = random_view(rng, dt, (57, 40, 9)).permute(1, 2, 0)                 # shape (40, 9, 57), strided
    m = rng.random((40, 9, 57)) < 0.35
    mask = View.from_numpy(m)
    offs_want = OI.mask_offsets(mask, a.strides)
    got, count = _mask_offsets_gpu(mask, a.strides)
    assert count == len(offs_want) and np.array_equal(got[:count], offs_want)
    lo, hi = 0, a.storage.size - itemsize(dt) - a.offset
    scalar = View(a.storage, dt, (), (), a.offset)
    out = View.empty(dt, (count,))
    dv = H.DeviceViews()
    offs_dev = _dev_i64(offs_want)
    ocn.gather(dv.tensor(scalar), offs_dev, lo, hi, dv.tensor(out))
    torch.cuda.synchronize()
    got_rows = dv.download(out).copy()
    OI.gather(scalar, offs_want, out, lo, hi)
    assert np.array_equal(got_rows, out.storage)
    # the same selection as NumPy sees it
    assert View(got_rows, dt, (count,), out.strides, 0).to_numpy().tobytes() == a.to_numpy()[m].tobytes()
    # scatter new values to the selected places
    vals = random_view(rng, dt, (count,))
    dv = H.DeviceViews()
    ocn.scatter(dv.tensor(vals), offs_dev, lo, hi, dv.tensor(scalar))
    torch.cuda.synchronize()
    got_a = dv.download(scalar).copy()
    OI.scatter(vals, offs_want, scalar, lo, hi)
    assert np.array_equal(got_a, a.storage)


@pytest.mark.parametrize("dt", ("int8", "int16", "float", "double", "cdouble"))
def test_single_elements_four_offsets_per_lane(dt):
    """Single elements with a contiguous rows side: lanes take four offsets at a time.  Counts
    that are not multiples of four, offsets outside the stated range inside a group of four
    (only that element is skipped), a rows side that starts off the alignment of a piece of
    four (the one-offset kernel), repeated offsets in a gather."""
    import torch
    import paper_1810_08723_amd as ocn
    es = itemsize(dt)
    rng = rng_for(17250 + es)
    src = random_view(rng, dt, (5000,))
    scalar = View(src.storage, dt, (), (), 0)
    for n in (1, 3, 4, 5, 1021, 1024, 4099):
        offs = rng.integers(0, 5000, size=n).astype(np.int64) * es
        lo, hi = 1000 * es, 3999 * es                      # about two in five are outside
        for skew in (0, 1):                                # rows side on / off a 4-element boundary
            base = View.empty(dt, (n + skew,))
            out = View(base.storage, dt, (n,), (es,), skew * es)
            dv = H.DeviceViews()
            ocn.gather(dv.tensor(scalar), _dev_i64(offs), lo, hi, dv.tensor(out))
            torch.cuda.synchronize()
            got = dv.download(out).copy()
            OI.gather(scalar, offs, out, lo, hi)
            assert np.array_equal(got, out.storage), (dt, n, skew)
            # scatter: unique in-range targets, others skipped
            perm = rng.permutation(5000)[:n].astype(np.int64) * es
            vals_base = random_view(rng, dt, (n + skew,))
            vals = View(vals_base.storage, dt, (n,), (es,), skew * es)
            target = random_view(rng, dt, (5000,))
            tscalar = View(target.storage, dt, (), (), 0)
            dv = H.DeviceViews()
            ocn.scatter(dv.tensor(vals), _dev_i64(perm), lo, hi, dv.tensor(tscalar))
            torch.cuda.synchronize()
            got_t = dv.download(tscalar).copy()
            OI.scatter(vals, perm, tscalar, lo, hi)
            assert np.array_equal(got_t, target.storage), (dt, n, skew)


def test_gather_rows_by_index_array_and_skipped_offsets():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17300)
    a = random_view(rng, "float", (300, 70, 6), specials=False)
    idx = rng.integers(-300, 300, size=(500,)).astype(np.int64)
    offs, bad = OI.index_offsets(idx, 300, a.strides[0])
    assert bad == 0
    inner = View(a.storage, "float", (70, 6), a.strides[1:], a.offset)
    for out in (View.empty("float", (500, 70, 6)), View.empty("float", (70, 500, 6)).permute(1, 0, 2)):
        dv = H.DeviceViews()
        ocn.gather(dv.tensor(inner), _dev_i64(offs), 0, 299 * a.strides[0], dv.tensor(out))
        torch.cuda.synchronize()
        got = dv.download(out).copy()
        OI.gather(inner, offs, out, 0, 299 * a.strides[0])
        assert np.array_equal(got, out.storage)
        assert np.array_equal(View(got, "float", out.sizes, out.strides, 0).to_numpy(), a.to_numpy()[idx])
    # index along the middle axis of the same tensor: the inner view is what is left of it
    idx2 = np.array([69, 0, -1, 5], dtype=np.int64)
    offs2, _ = OI.index_offsets(idx2, 70, a.strides[1])
    inner2 = View(a.storage, "float", (300, 6), (a.strides[0], a.strides[2]), a.offset)
    out = View.empty("float", (4, 300, 6))
    dv = H.DeviceViews()
    ocn.gather(dv.tensor(inner2), _dev_i64(offs2), 0, 69 * a.strides[1], dv.tensor(out))
    torch.cuda.synchronize()
    assert np.array_equal(View(dv.download(out), "float", out.sizes, out.strides, 0).to_numpy(),
                          np.moveaxis(a.to_numpy()[:, idx2, :], 1, 0))
    # offsets outside [lo, hi] are not followed: those rows keep their old contents
    offs3 = offs.copy()
    offs3[::7] = 10 ** 12
    offs3[3::7] = -8
    out = View.empty("float", (500, 70, 6))
    dv = H.DeviceViews()
    ocn.gather(dv.tensor(inner), _dev_i64(offs3), 0, 299 * a.strides[0], dv.tensor(out))
    torch.cuda.synchronize()
    got = dv.download(out).copy()
    OI.gather(inner, offs3, out, 0, 299 * a.strides[0])
    assert np.array_equal(got, out.storage)


def test_scatter_rows():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17301)
    a = random_view(rng, "int16", (200, 33))
    perm = rng.permutation(200)[:150].astype(np.int64)                    # distinct rows
    offs, _ = OI.index_offsets(perm, 200, a.strides[0])
    src = random_view(rng, "int16", (150, 33))
    inner = View(a.storage, "int16", (33,), a.strides[1:], a.offset)
    dv = H.DeviceViews()
    ocn.scatter(dv.tensor(src), _dev_i64(offs), 0, 199 * a.strides[0], dv.tensor(inner))
    torch.cuda.synchronize()
    got = dv.download(inner).copy()
    want = a.to_numpy().copy()
    want[perm] = src.to_numpy()
    OI.scatter(src, offs, inner, 0, 199 * a.strides[0])
    assert np.array_equal(got, a.storage) and np.array_equal(a.to_numpy(), want)


@pytest.mark.parametrize("dt,inner_len", [("float", 1), ("float", 3), ("float", 4), ("float", 12), ("float", 100),
                                          ("float", 256), ("float", 1028), ("int8", 48), ("int8", 50), ("half", 40),
                                          ("double", 6), ("cdouble", 5), ("cfloat", 34)])
def test_gather_scatter_row_lengths_and_alignments(dt, inner_len):
    # short rows share a workgroup, long rows take several; rows whose length, placement and
    # strides allow it move in 16-byte items, rows starting at other offsets element by element
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(17400 + inner_len + sum(map(ord, dt)))
    nrows, pick = 333, 777
    es = itemsize(dt)
    a = random_view(rng, dt, (nrows, inner_len))
    idx = rng.integers(0, nrows, size=(pick,)).astype(np.int64)
    offs, _ = OI.index_offsets(idx, nrows, a.strides[0])
    inner = View(a.storage, dt, (inner_len,), a.strides[1:], a.offset)
    out = View.empty(dt, (pick, inner_len))
    dv = H.DeviceViews()
    ocn.gather(dv.tensor(inner), _dev_i64(offs), 0, (nrows - 1) * a.strides[0], dv.tensor(out))
    torch.cuda.synchronize()
    got = dv.download(out).copy()
    OI.gather(inner, offs, out, 0, (nrows - 1) * a.strides[0])
    assert np.array_equal(got, out.storage)
    # window rows: overlapping windows of a long vector, starting at arbitrary elements
    vec = random_view(rng, dt, (5000,))
    starts = rng.integers(0, 5000 - inner_len, size=(pick,)).astype(np.int64)
    woffs = starts * es
    win = View(vec.storage, dt, (inner_len,), (es,), vec.offset)
    out2 = View.empty(dt, (pick, inner_len))
    dv = H.DeviceViews()
    ocn.gather(dv.tensor(win), _dev_i64(woffs), 0, (5000 - inner_len) * es, dv.tensor(out2))
    torch.cuda.synchronize()
    got2 = dv.download(out2).copy()
    OI.gather(win, woffs, out2, 0, (5000 - inner_len) * es)
    assert np.array_equal(got2, out2.storage)
    # scatter distinct rows back
    perm = rng.permutation(nrows)[:200].astype(np.int64)
    poffs, _ = OI.index_offsets(perm, nrows, a.strides[0])
    src = random_view(rng, dt, (200, inner_len))
    dv = H.DeviceViews()
    ocn.scatter(dv.tensor(src), _dev_i64(poffs), 0, (nrows - 1) * a.strides[0], dv.tensor(inner))
    torch.cuda.synchronize()
    got3 = dv.download(inner).copy()
    OI.scatter(src, poffs, inner, 0, (nrows - 1) * a.strides[0])
    assert np.array_equal(got3, a.storage)


@pytest.mark.parametrize("seed", range(10))
def test_fuzz_gather_scatter(seed):
    # random element types, inner shapes (0 to 3 dims, permuted), strided row tensors and offsets
    # (some outside the stated range): gather into a strided output, scatter of distinct rows
    import torch
    import paper_1810_08723_amd as ocn
    from workloads.fuzz import random_strided_view
    rng = rng_for(17500 + seed)
    types = ("int8", "int16", "half", "float", "double", "cfloat", "cdouble", "int64", "bool")
    for it in range(6):
        dt = types[int(rng.integers(0, len(types)))]
        es = itemsize(dt)
        nin = int(rng.integers(0, 4))
        inner_shape = tuple(int(rng.choice([1, 2, 3, 4, 5, 8, 16, 17, 33, 64])) for _ in range(nin))
        nrows = int(rng.integers(1, 60))
        full = random_view(rng, dt, (nrows,) + inner_shape)
        perm = [int(p) for p in rng.permutation(nin)] if nin else []
        inner = View(full.storage, dt, tuple(inner_shape[p] for p in perm), tuple(full.strides[1 + p] for p in perm),
                     full.offset)
        pick = int(rng.integers(0, 200))
        offs = rng.integers(0, nrows, size=(pick,)).astype(np.int64) * full.strides[0]
        if pick and rng.random() < 0.5:
            bad = rng.integers(0, pick, size=(max(1, pick // 7),))
            offs[bad] = rng.choice([-es, 10 ** 9, nrows * full.strides[0]], size=bad.shape)
        lo, hi = 0, (nrows - 1) * full.strides[0]
        out = random_strided_view(rng, dt, (pick,) + inner.sizes, writable=True)
        print("fuzz-gather", seed, it, dt, inner_shape, perm, pick, flush=True)
        dv = H.DeviceViews()
        ocn.gather(dv.tensor(inner), _dev_i64(offs), lo, hi, dv.tensor(out))
        torch.cuda.synchronize()
        got = dv.download(out).copy()
        OI.gather(inner, offs, out, lo, hi)
        assert np.array_equal(got, out.storage)
        k = int(rng.integers(0, nrows + 1))
        soffs = rng.permutation(nrows)[:k].astype(np.int64) * full.strides[0]
        src = random_strided_view(rng, dt, (k,) + inner.sizes, allow_broadcast=False)
        dv = H.DeviceViews()
        ocn.scatter(dv.tensor(src), _dev_i64(soffs), lo, hi, dv.tensor(inner))
        torch.cuda.synchronize()
        got = dv.download(inner).copy()
        OI.scatter(src, soffs, inner, lo, hi)
        assert np.array_equal(got, full.storage)
