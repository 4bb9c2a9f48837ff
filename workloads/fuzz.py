"""Random strided views for fuzz tests: permuted, stepped, reversed, broadcast and offset views
over dense seeded storage.  View construction only - none of the engine's arithmetic."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from .values import random_array
from .views import View, itemsize


def random_shape(rng: np.random.Generator, max_ndim: int = 5, max_elems: int = 6000) -> Tuple[int, ...]:
    ndim = int(rng.integers(0, max_ndim + 1))
    shape: List[int] = []
    total = 1
    for _ in range(ndim):
        kind = int(rng.integers(0, 6))
        s = (1 if kind == 0 else int(rng.integers(2, 6)) if kind == 1 else int(rng.integers(6, 40)) if kind <= 3
             else int(2 ** rng.integers(1, 7)) if kind == 4 else int(rng.integers(40, 130)))
        if total * s > max_elems:
            s = 1 + int(rng.integers(0, 2))
        shape.append(s)
        total *= s
    return tuple(shape)


def random_strided_view(rng: np.random.Generator, dtype: str, shape: Sequence[int],
                        specials: bool = True, allow_broadcast: bool = True,
                        writable: bool = False) -> View:
    """A view of the given logical shape over fresh seeded storage.

    Inputs may be broadcast (size-1 storage axes stretched with zero strides) and may drop
    leading axes; outputs (``writable``) never alias themselves."""
    shape = tuple(int(s) for s in shape)
    ndim = len(shape)
    perm = list(rng.permutation(ndim)) if ndim else []
    steps = [int(rng.choice([1, 1, 1, 2, 3])) for _ in range(ndim)]
    flips = [bool(rng.random() < 0.25) for _ in range(ndim)]
    bcast = [False] * ndim
    if allow_broadcast and not writable:
        bcast = [bool(rng.random() < 0.15) for _ in range(ndim)]
    # dense buffer in permuted axis order, each axis long enough for its step
    buf_shape = [0] * ndim
    for pos, ax in enumerate(perm):
        n = 1 if bcast[ax] else shape[ax]
        buf_shape[pos] = max(1, (n - 1) * steps[ax] + 1) if n > 0 else 1
    pad = int(rng.integers(0, 3)) * itemsize(dtype)
    arr = random_array(rng, dtype, tuple(buf_shape), specials)
    v = View.from_numpy(arr, dtype)
    if pad:  # shift the view inside a slightly larger storage
        storage = np.concatenate([np.full(pad, 0x5A, np.uint8), v.storage, np.full(pad, 0x5A, np.uint8)])
        v = View(storage, v.dtype, v.sizes, v.strides, v.offset + pad)
    inv = [0] * ndim
    for pos, ax in enumerate(perm):
        inv[ax] = pos
    if ndim:
        v = v.permute(*inv)  # logical axis order again
    for ax in range(ndim):
        n = 1 if bcast[ax] else shape[ax]
        v = v.slice(ax, 0, max(1, (n - 1) * steps[ax] + 1) if n > 0 else 0, steps[ax])
        if flips[ax] and n > 1:
            v = v.flip(ax)
    assert tuple(1 if bcast[ax] else shape[ax] for ax in range(ndim)) == v.sizes, (v.sizes, shape)
    if not writable and allow_broadcast:
        if rng.random() < 0.5:
            v = v.broadcast_to(shape)          # explicit zero strides
        else:
            while v.ndim and v.sizes[0] == 1 and rng.random() < 0.5:
                v = v.select(0, 0)             # lower rank: left-padded by the engine
    assert v.in_bounds()
    return v
