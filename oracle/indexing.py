"""CPU oracle of index binding, gather and scatter (section 3.2.2 of the paper: index arrays are
checked for validity and negative indices converted; boolean masks are counted and converted to
explicit indices; bound to strides, both become relative offsets into the data buffer, after
which indexed elements are copied out of, or into, the tensor).  TEST INFRASTRUCTURE ONLY.

Plain Python / NumPy loops over the definition; nothing here is shared with the GPU library.
Operands are ``workloads.views.View`` objects; offsets are NumPy int64 arrays of byte offsets
relative to element (0, ..., 0) of the tensor being indexed.
"""
from __future__ import annotations

import itertools
from typing import Sequence, Tuple

import numpy as np

from workloads.views import View, itemsize


def index_offsets(index: np.ndarray, dim_size: int, stride_bytes: int) -> Tuple[np.ndarray, int]:
    """Binds an index array to a dimension's size and stride: negative indices count from the
    end; indices outside [-dim_size, dim_size) are invalid (their offset is 0).  Returns the
    offsets, shaped like `index`, and the number of invalid indices."""
    out = np.zeros(index.shape, dtype=np.int64)
    invalid = 0
    for pos in np.ndindex(index.shape):
        i = int(index[pos])
        if i < 0:
            i += dim_size
        if 0 <= i < dim_size:
            out[pos] = i * stride_bytes
        else:
            invalid += 1
    return out, invalid


def mask_offsets(mask: View, target_strides: Sequence[int]) -> np.ndarray:
    """Offsets of the elements a boolean mask selects, in row-major order of the mask's own
    dimensions, bound to the byte strides of the tensor it will index."""
    m = mask.to_numpy()
    assert m.dtype == np.bool_ and len(target_strides) == m.ndim
    offs = []
    for idx in itertools.product(*[range(s) for s in m.shape]):
        if m[idx]:
            offs.append(sum(i * s for i, s in zip(idx, target_strides)))
    return np.array(offs, dtype=np.int64)


def _scalar_size(dtype: str) -> int:
    # a complex element is two scalars (section 3.1.3: each is stored in the tensor's byte order)
    return itemsize(dtype) // 2 if dtype in ("chalf", "cfloat", "cdouble") else itemsize(dtype)


def _move(dst_storage: np.ndarray, dst: int, src_storage: np.ndarray, src: int, dtype: str, reverse: bool) -> None:
    """Copies one element; `reverse`: the two tensors are stored in different byte orders
    (section 3.1.3), so every scalar of the element has its bytes reversed on the way."""
    es, sc = itemsize(dtype), _scalar_size(dtype)
    raw = src_storage[src:src + es].copy()
    if reverse and sc > 1:
        raw = raw.reshape(es // sc, sc)[:, ::-1].reshape(es)
    dst_storage[dst:dst + es] = raw


def _inner_offsets(view: View):
    for idx in itertools.product(*[range(s) for s in view.sizes]):
        yield idx, sum(i * s for i, s in zip(idx, view.strides))


def gather(a_inner: View, offsets: np.ndarray, out: View, lo: int, hi: int) -> None:
    """out[j, i...] = element of a at byte offset offsets[j] + inner offset of i...; `a_inner`
    describes one indexed sub-tensor (its element (0,...,0) at offset 0).  Offsets outside
    [lo, hi] are skipped (that output row is left untouched).  The two tensors may be stored in
    different byte orders (section 3.1.3): values, not bytes, are what is copied."""
    es = itemsize(a_inner.dtype)
    assert out.dtype == a_inner.dtype and out.sizes == (len(offsets),) + tuple(a_inner.sizes)
    for j, off in enumerate(offsets):
        off = int(off)
        if off < lo or off > hi:
            continue
        for idx, inner in _inner_offsets(a_inner):
            src = a_inner.offset + off + inner
            dst = out.offset + j * out.strides[0] + sum(i * s for i, s in zip(idx, out.strides[1:]))
            _move(out.storage, dst, a_inner.storage, src, a_inner.dtype, a_inner.byteswapped != out.byteswapped)


def scatter(src: View, offsets: np.ndarray, out_inner: View, lo: int, hi: int) -> None:
    """Element of out at byte offset offsets[j] + inner offset of i... = src[j, i...].  Offsets
    outside [lo, hi] are skipped.  Offsets that repeat make the result depend on order; the
    tests never repeat them."""
    es = itemsize(src.dtype)
    assert src.dtype == out_inner.dtype and src.sizes == (len(offsets),) + tuple(out_inner.sizes)
    for j, off in enumerate(offsets):
        off = int(off)
        if off < lo or off > hi:
            continue
        for idx, inner in _inner_offsets(out_inner):
            dst = out_inner.offset + off + inner
            s = src.offset + j * src.strides[0] + sum(i * t for i, t in zip(idx, src.strides[1:]))
            _move(out_inner.storage, dst, src.storage, s, src.dtype, src.byteswapped != out_inner.byteswapped)
