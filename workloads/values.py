"""Seeded value generators for test and benchmark inputs.

Only random draws and dtype packing live here: no casting rule, promotion rule or tensor
operation of the engine is implemented in this module.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from .views import DTYPES, View, is_complex

_INT_RANGE = {
    "int8": (-2 ** 7, 2 ** 7 - 1), "int16": (-2 ** 15, 2 ** 15 - 1),
    "int32": (-2 ** 31, 2 ** 31 - 1), "int64": (-2 ** 63, 2 ** 63 - 1),
    "uint8": (0, 2 ** 8 - 1), "uint16": (0, 2 ** 16 - 1),
    "uint32": (0, 2 ** 32 - 1), "uint64": (0, 2 ** 64 - 1),
}


def rng_for(seed: int) -> np.random.Generator:
    """The generator every synthetic input is drawn from: PCG64 seeded with ``seed``."""
    return np.random.Generator(np.random.PCG64(seed))


def _real_mix(rng: np.random.Generator, n: int, np_dtype, specials: bool) -> np.ndarray:
    """Floats of mixed magnitude: unit normals, small integers, large and tiny values."""
    kind = rng.integers(0, 5, size=n)
    x = rng.standard_normal(n)
    x = np.where(kind == 1, rng.integers(-300, 301, size=n).astype(np.float64), x)
    x = np.where(kind == 2, x * 1e5, x)
    x = np.where(kind == 3, x * 1e-6, x)
    x = np.where(kind == 4, np.ldexp(rng.standard_normal(n), rng.integers(-30, 40, size=n)), x)
    if specials and n > 0:
        pool = np.array([0.0, -0.0, 1.0, -1.0, 0.5, -0.5, 255.0, 256.0, -128.0, -129.0, 32767.0,
                         32767.5, 32768.0, -32768.0, -32768.5, -32769.0, 65504.0, 65519.9, 65520.0,
                         2.0 ** 24, 2.0 ** 24 + 1, 2.0 ** 31, -2.0 ** 31, 2.0 ** 31 - 0.5, 2.0 ** 32,
                         2.0 ** 63, -2.0 ** 63, 2.0 ** 64, 1e300, -1e300, 6e-8, 3e-8, 1e-40,
                         np.inf, -np.inf, np.nan, 0.999999, -0.999999, 2047.5, 2048.5, 4097.0])
        pick = rng.random(n) < 0.25
        x = np.where(pick, pool[rng.integers(0, pool.size, size=n)], x)
    with np.errstate(over="ignore", invalid="ignore"):
        return x.astype(np_dtype)


def random_array(rng: np.random.Generator, dtype: str, sizes: Sequence[int],
                 specials: bool = True) -> np.ndarray:
    """Random numpy array for one element type (``chalf``: float16 with a trailing axis 2)."""
    sizes = tuple(int(s) for s in sizes)
    n = int(np.prod(sizes, dtype=np.int64)) if sizes else 1
    nd = DTYPES[dtype][1]
    if dtype == "bool":
        return (rng.random(n) < 0.5).reshape(sizes)
    if dtype in _INT_RANGE:
        lo, hi = _INT_RANGE[dtype]
        kind = rng.integers(0, 3, size=n)
        small = rng.integers(max(lo, -100), min(hi, 100) + 1, size=n, dtype=np.int64)
        if dtype == "uint64":
            wide = rng.integers(0, 2 ** 64, size=n, dtype=np.uint64)
            out = np.where(kind == 0, small.astype(np.uint64), wide)
            edge = np.array([0, 1, 2 ** 63 - 1, 2 ** 63, 2 ** 64 - 1, 2 ** 32, 2 ** 53 + 1], dtype=np.uint64)
        else:
            wide = rng.integers(lo, hi, size=n, dtype=np.int64, endpoint=True)
            out = np.where(kind == 0, small, wide)
            edge = np.array([lo, hi, 0, 1, min(hi, 127), max(lo, -128)], dtype=np.int64)
        if specials and n > 0:
            pick = kind == 2
            out = np.where(pick, edge[rng.integers(0, edge.size, size=n)], out)
        return out.astype(nd).reshape(sizes)
    if is_complex(dtype):
        comp = {"chalf": np.float16, "cfloat": np.float32, "cdouble": np.float64}[dtype]
        re = _real_mix(rng, n, comp, specials)
        im = _real_mix(rng, n, comp, specials)
        if dtype == "chalf":
            return np.stack([re, im], axis=-1).reshape(sizes + (2,))
        return _pack_complex(re, im, nd).reshape(sizes)
    return _real_mix(rng, n, nd, specials).reshape(sizes)


def _pack_complex(re: np.ndarray, im: np.ndarray, nd) -> np.ndarray:
    """Interleave components without arithmetic (re + 1j*im would turn inf+nan into nan)."""
    out = np.empty(re.shape, dtype=nd)
    out.real = re
    out.imag = im
    return out


def random_view(rng: np.random.Generator, dtype: str, sizes: Sequence[int],
                specials: bool = True) -> View:
    return View.from_numpy(random_array(rng, dtype, sizes, specials), dtype)
