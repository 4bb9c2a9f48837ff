"""ctypes binding of the CPU oracle (oracle/libocn_oracle.so).  TEST INFRASTRUCTURE ONLY.

Operands are ``workloads.views.View`` objects over host numpy storage.  Results are written
into the output view's storage in place.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

import numpy as np

from . import build as _build

MAX_DIMS = 8

DTYPE_CODE = {name: i for i, name in enumerate(
    ["bool", "int8", "int16", "int32", "int64", "uint8", "uint16", "uint32", "uint64",
     "half", "float", "double", "chalf", "cfloat", "cdouble"])}
DTYPE_NAME = {v: k for k, v in DTYPE_CODE.items()}

UNARY = {name: i for i, name in enumerate(["ident", "neg", "abs", "conj", "lnot", "bnot", "sqrt",
                                           "sin", "cos", "tan", "exp", "log", "bswap",
                                           "asin", "acos", "atan", "sinh", "cosh", "tanh"])}
BINARY = {name: i for i, name in enumerate(
    ["add", "sub", "mul", "div", "min", "max", "band", "bor", "bxor", "land", "lor", "lxor",
     "eq", "ne", "lt", "le", "gt", "ge", "absgt"])}
REDUCE = {name: i for i, name in enumerate(["sum", "prod", "min", "max", "any", "all"])}

ERR_DTYPE, ERR_SHAPE, ERR_EMPTY = -2, -4, -10
STRICT_TYPES = 1


class OrcTensor(C.Structure):
    _fields_ = [("base", C.c_void_p), ("offset", C.c_int64), ("dtype", C.c_int32),
                ("ndim", C.c_int32), ("size", C.c_int64 * MAX_DIMS),
                ("stride", C.c_int64 * MAX_DIMS), ("device", C.c_int32), ("byteswapped", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        P = C.POINTER(OrcTensor)
        L.orc_unary.argtypes = [C.c_int, P, P, C.c_uint32]
        L.orc_binary.argtypes = [C.c_int, P, P, P, C.c_uint32]
        L.orc_cast_copy.argtypes = [P, P]
        L.orc_reduce.argtypes = [C.c_int, P, C.POINTER(C.c_int32), C.c_int32, P]
        L.orc_promote.argtypes = [C.c_int, C.c_int]
        L.orc_dtype_size.argtypes = [C.c_int]
        L.orc_half_bits_to_double.argtypes = [C.c_uint16]
        L.orc_half_bits_to_double.restype = C.c_double
        L.orc_double_to_half_bits.argtypes = [C.c_double]
        L.orc_double_to_half_bits.restype = C.c_uint16
        _lib = L
    return _lib


def _desc(view) -> OrcTensor:
    assert view.storage.dtype == np.uint8 and view.storage.flags.c_contiguous
    assert view.ndim <= MAX_DIMS
    assert view.in_bounds(), "view reaches outside its storage"
    t = OrcTensor()
    t.base = view.storage.ctypes.data
    t.offset = view.offset
    t.dtype = DTYPE_CODE[view.dtype]
    t.ndim = view.ndim
    for d in range(view.ndim):
        t.size[d] = view.sizes[d]
        t.stride[d] = view.strides[d]
    t.device = -1
    t.byteswapped = 1 if getattr(view, "byteswapped", False) else 0
    return t


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _check(rc: int) -> None:
    if rc != 0:
        raise OracleError(rc)


def unary(op: str, a, out, flags: int = 0) -> None:
    _check(lib().orc_unary(UNARY[op], C.byref(_desc(a)), C.byref(_desc(out)), flags))


def binary(op: str, a, b, out, flags: int = 0) -> None:
    _check(lib().orc_binary(BINARY[op], C.byref(_desc(a)), C.byref(_desc(b)),
                            C.byref(_desc(out)), flags))


def cast_copy(src, dst) -> None:
    _check(lib().orc_cast_copy(C.byref(_desc(src)), C.byref(_desc(dst))))


def reduce(op: str, a, axes: Sequence[int], out) -> None:
    ax = (C.c_int32 * max(len(axes), 1))(*axes)
    _check(lib().orc_reduce(REDUCE[op], C.byref(_desc(a)), ax, len(axes), C.byref(_desc(out))))


def binary_reduce(ew_op: str, red_op: str, a, b, axes: Sequence[int], out, mid_dtype: str) -> None:
    """Reduction of an elementwise result (sections 3.2 and 5 of the paper: elementwise
    functions followed by a reduction along axes, as in the norm of the QR example), written
    out as its definition: materialise binary(ew_op, a, b) as a tensor of type `mid_dtype`
    and the broadcast shape, then reduce it over `axes` into `out`.  Nothing is fused here."""
    from workloads.views import View
    shape = tuple(int(s) for s in np.broadcast_shapes(tuple(a.sizes), tuple(b.sizes)))
    mid = View.empty(mid_dtype, shape)
    binary(ew_op, a, b, mid)
    reduce(red_op, mid, axes, out)


def domain_check(op: str, a) -> bool:
    """Compute modes (section 3.2.1: warning, error and complex modes check the elements against
    the operator's domain first): True if some element of `a` lies outside the real domain of
    `op` - negative for sqrt and log, of magnitude above one for asin and acos (the paper's own
    example); the other operations are defined everywhere.  NaNs do not count.  Written as its
    definition: any(a < 0), any(|a| > |1|), through the elementwise and reduction oracle."""
    from workloads.views import View
    out = View.empty("bool", ())
    if op in ("sqrt", "log"):
        zero = View(np.zeros(16, dtype=np.uint8), a.dtype, (), (), 0)
        binary_reduce("lt", "any", a, zero, list(range(a.ndim)), out, "bool")
    elif op in ("asin", "acos"):
        one = View.empty(a.dtype, ())
        cast_copy(View.from_numpy(np.array(1, dtype=np.int8)), one)
        binary_reduce("absgt", "any", a, one, list(range(a.ndim)), out, "bool")
    else:
        return False
    return bool(out.to_numpy())


MODES = ("standard", "warning", "error", "complex")


class DomainError(ValueError):
    """Error mode: some element lies outside the operator's domain."""


def unary_mode(op: str, mode: str, a, out, out_complex=None) -> dict:
    """A unary operation in one of the paper's compute modes (section 3.2.1), written as its
    definition on top of the domain check and the plain operation:
      standard  no check; NaN where an element is outside the domain;
      warning   check, then compute as in standard mode; the caller is told (`outside`);
      error     check; outside the domain nothing is computed and DomainError is raised;
      complex   check; outside the domain the result is computed in the complex type of
                `out_complex` (the real input converts with a zero imaginary part) and written
                there, otherwise in `out` as usual.
    Returns {"outside": None (not checked) | bool, "wrote": "out" | "out_complex"}."""
    assert mode in MODES
    if mode == "standard":
        unary(op, a, out)
        return {"outside": None, "wrote": "out"}
    outside = domain_check(op, a)
    if mode == "error" and outside:
        raise DomainError(op)
    if mode == "complex" and outside:
        unary(op, a, out_complex)
        return {"outside": True, "wrote": "out_complex"}
    unary(op, a, out)
    return {"outside": outside, "wrote": "out"}


def promote(a: str, b: str) -> str:
    return DTYPE_NAME[lib().orc_promote(DTYPE_CODE[a], DTYPE_CODE[b])]


def half_bits_to_double(h: int) -> float:
    return lib().orc_half_bits_to_double(h)


def double_to_half_bits(x: float) -> int:
    return lib().orc_double_to_half_bits(x)
