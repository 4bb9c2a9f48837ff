"""Runs one operation through the GPU library and through the CPU oracle on the same seeded
views and compares the complete output storage, byte for byte (NaN payloads excepted)."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

from workloads.views import DTYPES, View, itemsize

_FLOAT_COMPONENT = {"half": np.float16, "float": np.float32, "double": np.float64,
                    "chalf": np.float16, "cfloat": np.float32, "cdouble": np.float64}


class DeviceViews:
    """Uploads the storages behind a set of views once each (views sharing storage keep sharing it)."""

    def __init__(self, device: int = 0):
        import torch
        self.torch = torch
        self.device = device
        self._by_id: Dict[int, object] = {}

    def tensor(self, view: View):
        import paper_1810_08723_amd as ocn
        key = id(view.storage)
        if key not in self._by_id:
            host = view.storage if view.storage.size else np.zeros(1, dtype=np.uint8)
            # keep the host array alive too: a freed array's id could be handed out again
            self._by_id[key] = (view.storage, self.torch.from_numpy(host.copy()).to(f"cuda:{self.device}"))
        assert self._by_id[key][0] is view.storage
        assert view.in_bounds()
        return ocn.Tensor.on_storage(self._by_id[key][1], view.dtype, view.sizes, view.strides, view.offset,
                                     getattr(view, "byteswapped", False))

    def download(self, view: View) -> np.ndarray:
        got = self._by_id[id(view.storage)][1].cpu().numpy()
        return got[:view.storage.size]


_SCALAR_BYTES = {"int16": 2, "uint16": 2, "half": 2, "chalf": 2, "int32": 4, "uint32": 4, "float": 4, "cfloat": 4,
                 "int64": 8, "uint64": 8, "double": 8, "cdouble": 8}


def native_order(dtype: str, storage: np.ndarray) -> np.ndarray:
    """The bytes of a storage that holds scalars of `dtype` in the other byte order, every scalar
    reversed back (the storage must consist of such scalars from its first byte on)."""
    sb = _SCALAR_BYTES.get(dtype, 1)
    n = storage.size // sb * sb
    if sb == 1:
        return storage
    return np.concatenate([storage[:n].reshape(-1, sb)[:, ::-1].reshape(-1), storage[n:]])


def storages_equal(dtype: str, got: np.ndarray, want: np.ndarray, swapped: bool = False) -> bool:
    """Byte equality; where the bytes differ, both sides must hold NaN in the same float slot.
    `swapped`: both storages hold their scalars in the other byte order."""
    if np.array_equal(got, want):
        return True
    if swapped:
        got, want = native_order(dtype, got), native_order(dtype, want)
    if dtype not in _FLOAT_COMPONENT:
        return False
    comp = np.dtype(_FLOAT_COMPONENT[dtype])
    n = got.size // comp.itemsize * comp.itemsize
    if not np.array_equal(got[n:], want[n:]):
        return False
    # Float slots are aligned to the component size relative to the storage start in all the
    # tests that use this helper.
    g = got[:n].view(comp)
    w = want[:n].view(comp)
    gi = got[:n].view({2: np.uint16, 4: np.uint32, 8: np.uint64}[comp.itemsize])
    wi = want[:n].view(gi.dtype)
    diff = gi != wi
    return bool(np.all(np.isnan(g[diff]) & np.isnan(w[diff])))


def first_mismatch(dtype: str, got: np.ndarray, want: np.ndarray) -> str:
    idx = np.nonzero(got != want)[0]
    if idx.size == 0:
        return "no byte differs"
    i = int(idx[0])
    lo = max(0, i - 8)
    return (f"{idx.size} bytes differ; first at byte {i}: got {got[lo:i + 16].tolist()} "
            f"want {want[lo:i + 16].tolist()}")


def check_binary(op: str, a: View, b: View, out: View, flags: int = 0) -> None:
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = DeviceViews()
    ta, tb, to = dv.tensor(a), dv.tensor(b), dv.tensor(out)
    ocn.binary(op, ta, tb, to, flags)
    dv.torch.cuda.synchronize()
    got = dv.download(out)
    O.binary(op, a, b, out, flags)          # oracle writes into the host storage
    assert storages_equal(out.dtype, got, out.storage, out.byteswapped), first_mismatch(out.dtype, got, out.storage)


def check_unary(op: str, a: View, out: View, flags: int = 0) -> None:
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = DeviceViews()
    ta, to = dv.tensor(a), dv.tensor(out)
    ocn.unary(op, ta, to, flags)
    dv.torch.cuda.synchronize()
    got = dv.download(out)
    O.unary(op, a, out, flags)
    assert storages_equal(out.dtype, got, out.storage, out.byteswapped), first_mismatch(out.dtype, got, out.storage)


def run_reduce(op: str, a: View, axes: Sequence[int], out: View):
    """Returns (gpu storage, oracle storage) of out after the reduction."""
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = DeviceViews()
    ta, to = dv.tensor(a), dv.tensor(out)
    ocn.reduce(op, ta, list(axes), to)
    dv.torch.cuda.synchronize()
    got = dv.download(out)
    O.reduce(op, a, list(axes), out)
    return got, out.storage


def run_binary_reduce(ew_op: str, red_op: str, a: View, b: View, axes: Sequence[int], out: View, mid_dtype: str):
    """Returns (gpu storage, oracle storage) of out after reduce(red_op, binary(ew_op, a, b))."""
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = DeviceViews()
    ta, tb, to = dv.tensor(a), dv.tensor(b), dv.tensor(out)
    ocn.binary_reduce(ew_op, red_op, ta, tb, list(axes), to, mid_dtype)
    dv.torch.cuda.synchronize()
    got = dv.download(out)
    O.binary_reduce(ew_op, red_op, a, b, list(axes), out, mid_dtype)
    return got, out.storage


def plan_reduce(op: str, a: View, axes: Sequence[int], out: View) -> dict:
    """The planner's decision for a reduction (no launch; stand-in base addresses)."""
    import paper_1810_08723_amd as ocn
    ta = ocn.Tensor(1 << 40, a.dtype, a.sizes, a.strides, a.offset, 0)
    to = ocn.Tensor(1 << 41, out.dtype, out.sizes, out.strides, out.offset, 0)
    return ocn.plan_reduce(op, ta, list(axes), to)
