"""Argument checks of the index binding, gather and scatter entry points: every documented
error is reported before anything is launched (so these run without a GPU)."""
import ctypes as C

import numpy as np
import pytest

import paper_1810_08723_amd as ocn
from paper_1810_08723_amd import binding as B

E = B.ERR


def t(dtype, sizes, strides=None, base=0x100000000, offset=0):
    es = ocn.dtype_size(dtype)
    if strides is None:
        strides, acc = [], es
        for n in reversed(sizes):
            strides.insert(0, acc)
            acc *= n
    return ocn.Tensor(base, dtype, tuple(sizes), tuple(strides), offset, 0)


def test_index_offsets_errors():
    L = B.lib()
    idx, off = t("int64", (10,)), t("int64", (10,), base=0x200000000)
    cnt = C.c_void_p(0x300000000)
    call = lambda i, o, n=64, c=cnt: L.ocn_index_offsets(C.byref(i.desc()), n, 8, C.byref(o.desc()), c, None)
    assert call(t("int32", (10,)), off) == E["DTYPE"]
    assert call(idx, t("int64", (11,))) == E["SHAPE"]
    assert call(idx, t("int64", (10, 1))) == E["SHAPE"]
    assert call(idx, off, n=-1) == E["SHAPE"]
    assert call(idx, off, c=None) == E["NULLPTR"]
    assert call(t("int64", (10,), offset=4), off) == E["ALIGN"]


def test_mask_offsets_errors():
    L = B.lib()
    mask = t("bool", (100, 50))
    strides = (C.c_int64 * 2)(200, 4)
    offs, cnt, ws = C.c_void_p(0x200000000), C.c_void_p(0x300000000), C.c_void_p(0x400000000)
    need = L.ocn_mask_offsets_workspace_bytes(C.byref(mask.desc()))
    assert need >= 8 * (100 * 50 // 4096 + 1)
    call = lambda m, s=strides, o=offs, c=cnt, w=ws, wb=need: L.ocn_mask_offsets(C.byref(m.desc()), s, o, 5000, c, w, wb, None)
    assert call(t("uint8", (100, 50))) == E["DTYPE"]
    assert call(mask, s=None) == E["NULLPTR"]
    assert call(mask, c=None) == E["NULLPTR"]
    assert call(mask, o=None) == E["NULLPTR"]
    assert call(mask, w=None) == E["WORKSPACE"]
    assert call(mask, wb=need - 1) == E["WORKSPACE"]
    assert call(t("bool", (1 << 16, 1 << 15))) == E["SHAPE"]          # 2^31 elements: too many for one call
    assert call(mask, o=C.c_void_p(0x200000004)) == E["ALIGN"]


def test_gather_scatter_errors():
    L = B.lib()
    inner = t("float", (70, 6))
    rows = t("float", (500, 70, 6), base=0x200000000)
    offs = C.c_void_p(0x300000000)
    g = lambda a, o, n=500, of=offs: L.ocn_gather(C.byref(a.desc()), of, n, 0, 1 << 20, C.byref(o.desc()), None)
    assert g(inner, t("double", (500, 70, 6))) == E["DTYPE"]
    assert g(inner, t("float", (500, 70, 5))) == E["SHAPE"]
    assert g(inner, t("float", (500, 70))) == E["SHAPE"]
    assert g(inner, rows, n=499) == E["SHAPE"]
    assert g(inner, rows, of=None) == E["NULLPTR"]
    assert g(inner, rows, of=C.c_void_p(0x300000004)) == E["ALIGN"]
    assert g(t("float", (70, 6), strides=(24, 2)), rows) == E["ALIGN"]
    assert L.ocn_scatter(C.byref(rows.desc()), offs, 500, 0, 1 << 20, C.byref(t("half", (70, 6)).desc()), None) == E["DTYPE"]
    # nothing to do: success without touching anything
    assert g(inner, t("float", (0, 70, 6)), n=0) == B.OK
