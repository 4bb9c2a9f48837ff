"""Strided tensor views over raw byte storage, for building test and benchmark inputs.

A ``View`` is the tensor model of the Ocean paper (section 3.1.3 "Tensors": a data type,
up to eight dimensions, sizes and general strides given in bytes) laid over a flat byte
buffer ("Storage", section 3.1.2).  This module only *describes* memory: it creates
storage, and derives views by the basic-indexing rules of section 3.2.2 (ranges with
steps, reversed ranges, axis permutation, broadcasting through zero strides).  It holds
none of the engine's arithmetic - no casting rules, no promotion, no reductions and no
dimension canonicalisation - so both the CPU oracle's tests and the GPU tests can draw
their inputs from it.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Sequence, Tuple

import numpy as np

MAX_DIMS = 8  # section 3.1.3: at most eight tensor dimensions

# dtype name -> (element size in bytes, numpy dtype of one element or of one component)
# The fifteen element types are those of the footnote in section 4.
DTYPES = {
    "bool": (1, np.dtype(np.bool_)),
    "int8": (1, np.dtype(np.int8)),
    "int16": (2, np.dtype(np.int16)),
    "int32": (4, np.dtype(np.int32)),
    "int64": (8, np.dtype(np.int64)),
    "uint8": (1, np.dtype(np.uint8)),
    "uint16": (2, np.dtype(np.uint16)),
    "uint32": (4, np.dtype(np.uint32)),
    "uint64": (8, np.dtype(np.uint64)),
    "half": (2, np.dtype(np.float16)),
    "float": (4, np.dtype(np.float32)),
    "double": (8, np.dtype(np.float64)),
    "chalf": (4, np.dtype(np.float16)),  # two float16 components; numpy has no such scalar
    "cfloat": (8, np.dtype(np.complex64)),
    "cdouble": (16, np.dtype(np.complex128)),
}
DTYPE_NAMES = tuple(DTYPES)


def itemsize(dtype: str) -> int:
    return DTYPES[dtype][0]


def is_complex(dtype: str) -> bool:
    return dtype in ("chalf", "cfloat", "cdouble")


@dataclass(frozen=True)
class View:
    """dtype + sizes + byte strides + byte offset over a shared 1-D uint8 storage array."""

    storage: np.ndarray  # 1-D uint8, shared between views derived from one another
    dtype: str
    sizes: Tuple[int, ...]
    strides: Tuple[int, ...]  # bytes; may be zero or negative
    offset: int = 0  # bytes from storage start to element (0,...,0)
    byteswapped: bool = False  # the storage holds every scalar in the other byte order (section 3.1.3)

    # ---- construction -------------------------------------------------------------
    @staticmethod
    def empty(dtype: str, sizes: Sequence[int], order: str = "C", fill: int = 0xA5,
              pad_bytes: int = 0) -> "View":
        """New storage filled with a sentinel byte, viewed contiguously (row- or column-major)."""
        es = itemsize(dtype)
        sizes = tuple(int(s) for s in sizes)
        n = int(np.prod(sizes, dtype=np.int64)) if sizes else 1
        storage = np.full(n * es + 2 * pad_bytes, fill, dtype=np.uint8)
        strides = contiguous_strides(sizes, es, order)
        return View(storage, dtype, sizes, strides, pad_bytes)

    @staticmethod
    def from_numpy(arr: np.ndarray, dtype: str | None = None) -> "View":
        """Contiguous row-major view holding a copy of ``arr``.

        For ``chalf`` pass a float16 array whose last axis has length 2 (re, im).
        """
        if dtype is None:
            for name, (_, nd) in DTYPES.items():
                if name != "chalf" and nd == arr.dtype:
                    dtype = name
                    break
            else:
                raise TypeError(f"no element type for numpy dtype {arr.dtype}")
        if dtype == "chalf":
            assert arr.dtype == np.float16 and arr.shape[-1] == 2
            sizes = arr.shape[:-1]
        else:
            assert arr.dtype == DTYPES[dtype][1], (arr.dtype, dtype)
            sizes = arr.shape
        data = np.ascontiguousarray(arr)
        storage = data.reshape(-1).view(np.uint8).copy()
        return View(storage, dtype, tuple(sizes), contiguous_strides(sizes, itemsize(dtype), "C"), 0)

    # ---- derived views (all share storage) -----------------------------------------
    @property
    def ndim(self) -> int:
        return len(self.sizes)

    @property
    def numel(self) -> int:
        n = 1
        for s in self.sizes:
            n *= s
        return n

    def permute(self, *perm: int) -> "View":
        """view.dim[i] = self.dim[perm[i]] (axis manipulation without data movement)."""
        assert sorted(perm) == list(range(self.ndim))
        return replace(self, sizes=tuple(self.sizes[p] for p in perm),
                       strides=tuple(self.strides[p] for p in perm))

    def slice(self, axis: int, start: int, stop: int, step: int = 1) -> "View":
        """Range indexing along one axis with Python slice semantics (step may be negative)."""
        idx = range(*slice(start, stop, step).indices(self.sizes[axis]))
        n = len(idx)
        first = idx[0] if n else 0
        sizes = list(self.sizes)
        strides = list(self.strides)
        sizes[axis] = n
        strides[axis] = self.strides[axis] * step
        return replace(self, sizes=tuple(sizes), strides=tuple(strides),
                       offset=self.offset + first * self.strides[axis])

    def flip(self, axis: int) -> "View":
        """Reverse one axis: negative stride, offset moved to the last element."""
        n = self.sizes[axis]
        strides = list(self.strides)
        strides[axis] = -strides[axis]
        off = self.offset + (n - 1) * self.strides[axis] if n > 0 else self.offset
        return replace(self, strides=tuple(strides), offset=off)

    def select(self, axis: int, index: int) -> "View":
        """Scalar indexing along one axis: drops the axis."""
        if index < 0:
            index += self.sizes[axis]
        sizes = self.sizes[:axis] + self.sizes[axis + 1:]
        strides = self.strides[:axis] + self.strides[axis + 1:]
        return replace(self, sizes=sizes, strides=strides,
                       offset=self.offset + index * self.strides[axis])

    def broadcast_to(self, sizes: Sequence[int]) -> "View":
        """Stretch size-1 axes (and prepend axes) with zero strides."""
        sizes = tuple(int(s) for s in sizes)
        lead = len(sizes) - self.ndim
        assert lead >= 0
        strides = [0] * lead
        for s_new, s_old, st in zip(sizes[lead:], self.sizes, self.strides):
            if s_old == s_new:
                strides.append(st)
            else:
                assert s_old == 1, (self.sizes, sizes)
                strides.append(0)
        return replace(self, sizes=sizes, strides=tuple(strides))

    def unsqueeze(self, axis: int, stride: int = 0) -> "View":
        sizes = self.sizes[:axis] + (1,) + self.sizes[axis:]
        strides = self.strides[:axis] + (stride,) + self.strides[axis:]
        return replace(self, sizes=sizes, strides=strides)

    def reinterpret(self, dtype: str, extra_offset: int = 0) -> "View":
        """Another element type superimposed on the same storage, same sizes and strides
        (section 3.1.2: e.g. the imaginary part of a complex double tensor is a double
        view on the same storage)."""
        return replace(self, dtype=dtype, offset=self.offset + extra_offset)

    def with_storage(self, storage: np.ndarray) -> "View":
        assert storage.dtype == np.uint8 and storage.ndim == 1 and storage.size == self.storage.size
        return replace(self, storage=storage)

    def fresh_copy(self) -> "View":
        """Same descriptor over a private copy of the storage bytes."""
        return replace(self, storage=self.storage.copy())

    # ---- byte extent --------------------------------------------------------------
    def byte_range(self) -> Tuple[int, int]:
        """[lo, hi) of storage bytes touched by the view (lo == hi when it has no elements)."""
        if self.numel == 0:
            return (self.offset, self.offset)
        lo = hi = self.offset
        for n, st in zip(self.sizes, self.strides):
            if st < 0:
                lo += (n - 1) * st
            else:
                hi += (n - 1) * st
        return (lo, hi + itemsize(self.dtype))

    def in_bounds(self) -> bool:
        lo, hi = self.byte_range()
        return 0 <= lo and hi <= self.storage.size

    # ---- materialisation through numpy's own strided views (used only as a cross-check
    # of element addressing; never for arithmetic) -----------------------------------
    def to_numpy(self) -> np.ndarray:
        """Gather the viewed elements into a new contiguous row-major numpy array.

        ``chalf`` comes back as float16 with a trailing axis of length 2.
        """
        assert self.in_bounds()
        _, nd = DTYPES[self.dtype]
        shape, strides = self.sizes, self.strides
        if self.dtype == "chalf":
            shape, strides = shape + (2,), strides + (2,)
        if self.numel == 0:
            return np.zeros(shape, dtype=nd)
        v = np.ndarray(shape, dtype=nd, buffer=self.storage, offset=self.offset, strides=strides)
        out = np.array(v, order="C")
        return out.byteswap() if self.byteswapped else out     # numpy reverses each scalar's bytes

    def in_other_byte_order(self) -> "View":
        """A copy of the viewed storage with the bytes of every scalar reversed, described by the
        same sizes, strides and offset and flagged as stored in the other byte order: it holds
        the same values as ``self``."""
        _, nd = DTYPES[self.dtype]
        sb = nd.itemsize if self.dtype not in ("cfloat", "cdouble") else nd.itemsize // 2
        storage = self.storage.copy()
        if sb > 1:
            # reverse, in place, the scalars this view addresses (other bytes of the storage stay)
            shape, strides = self.sizes, self.strides
            comp = np.dtype(f"V{sb}")
            ncomp = itemsize(self.dtype) // sb
            if ncomp > 1:
                shape, strides = shape + (ncomp,), strides + (sb,)
            if self.numel:
                v = np.ndarray(shape, dtype=comp, buffer=storage, offset=self.offset, strides=strides)
                raw = np.array(v, order="C").view(np.uint8).reshape(shape + (sb,))[..., ::-1]
                v[...] = np.ascontiguousarray(raw).view(comp).reshape(shape)
        return replace(self, storage=storage, byteswapped=not self.byteswapped)


def contiguous_strides(sizes: Sequence[int], es: int, order: str = "C") -> Tuple[int, ...]:
    """Byte strides of a dense layout: "C" = last axis fastest, "F" = first axis fastest
    (the paper's default layout is column-major, section 3.1.3)."""
    n = len(sizes)
    strides = [0] * n
    acc = es
    axes = range(n - 1, -1, -1) if order == "C" else range(n)
    for ax in axes:
        strides[ax] = acc
        acc *= max(int(sizes[ax]), 1)
    return tuple(strides)
