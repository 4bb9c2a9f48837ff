"""Per-index brute-force evaluation of whole operations over views, in pure Python, built on
tests/exactmath.py.  Used to pin the CPU oracle on tiny tensors."""
from __future__ import annotations

import itertools

import numpy as np

import exactmath as X
from workloads.views import View, itemsize


def _addr(view: View, idx, lead: int = 0) -> int:
    off = view.offset
    for d in range(view.ndim):
        i = 0 if view.sizes[d] == 1 else idx[lead + d]
        off += i * view.strides[d]
    return off


def _load(view: View, off: int):
    es = itemsize(view.dtype)
    return X.decode(view.dtype, bytes(view.storage[off:off + es]))


def _store(storage: np.ndarray, dt: str, off: int, v) -> None:
    raw = X.encode(dt, v)
    storage[off:off + len(raw)] = np.frombuffer(raw, dtype=np.uint8)


def binary(op: str, a: View, b: View, out: View) -> np.ndarray:
    """Expected bytes of out.storage after out = a (op) b."""
    T = X.compute_type(op, a.dtype, b.dtype, out.dtype)
    assert X.binary_supported(op, T)
    res = out.storage.copy()
    la, lb = out.ndim - a.ndim, out.ndim - b.ndim
    for idx in itertools.product(*[range(s) for s in out.sizes]):
        va = X.convert(_load(a, _addr(a, idx, la)), a.dtype, T)
        vb = X.convert(_load(b, _addr(b, idx, lb)), b.dtype, T)
        r = X.apply_binary(op, T, va, vb)
        rt = T if (op in X.ARITH or op in X.BITWISE) else "bool"
        _store(res, out.dtype, _addr(out, idx), X.convert(r, rt, out.dtype))
    return res


def unary(op: str, a: View, out: View) -> np.ndarray:
    T = "bool" if op == "lnot" else out.dtype
    assert X.unary_supported(op, T)
    res = out.storage.copy()
    la = out.ndim - a.ndim
    for idx in itertools.product(*[range(s) for s in out.sizes]):
        va = X.convert(_load(a, _addr(a, idx, la)), a.dtype, T)
        r = X.apply_unary(op, T, va)
        _store(res, out.dtype, _addr(out, idx), X.convert(r, T, out.dtype))
    return res


def storages_match(dt: str, got: np.ndarray, want: np.ndarray, view: View | None = None) -> bool:
    """Byte equality of two storages; floating elements of ``view`` may differ in NaN payload."""
    if np.array_equal(got, want):
        return True
    if view is None or X.kind(dt) not in "fc":
        return False
    touched = np.zeros(got.size, dtype=bool)
    es = itemsize(dt)
    for idx in itertools.product(*[range(s) for s in view.sizes]):
        off = _addr(view, idx)
        touched[off:off + es] = True
        if not X.same_value(dt, bytes(got[off:off + es]), bytes(want[off:off + es])):
            return False
    return bool(np.array_equal(got[~touched], want[~touched]))
