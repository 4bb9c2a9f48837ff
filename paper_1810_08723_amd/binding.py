"""Thin ctypes binding of libocn.so - argument marshalling only.

Every step of every operation runs inside the library's HIP kernels; nothing here computes.
PyTorch appears only as the owner of device memory and streams.  If the built library is
missing the import fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Any, Optional, Sequence, Tuple

MAX_DIMS = 8
HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libocn.so")

DTYPES = ("bool", "int8", "int16", "int32", "int64", "uint8", "uint16", "uint32", "uint64",
          "half", "float", "double", "chalf", "cfloat", "cdouble")
DTYPE_CODE = {n: i for i, n in enumerate(DTYPES)}
UNARY_OPS = ("ident", "neg", "abs", "conj", "lnot", "bnot", "sqrt", "sin", "cos", "tan", "exp", "log", "bswap",
             "asin", "acos", "atan", "sinh", "cosh", "tanh")
BINARY_OPS = ("add", "sub", "mul", "div", "min", "max", "band", "bor", "bxor", "land", "lor",
              "lxor", "eq", "ne", "lt", "le", "gt", "ge", "absgt")
REDUCE_OPS = ("sum", "prod", "min", "max", "any", "all")
UNARY_CODE = {n: i for i, n in enumerate(UNARY_OPS)}
BINARY_CODE = {n: i for i, n in enumerate(BINARY_OPS)}
REDUCE_CODE = {n: i for i, n in enumerate(REDUCE_OPS)}

STRICT_TYPES = 1

OK = 0
ERR = {"NULLPTR": -1, "DTYPE": -2, "NDIM": -3, "SHAPE": -4, "DEVICE": -5, "ALIGN": -6,
       "OVERLAP_OUT": -7, "ALIAS": -8, "WORKSPACE": -9, "EMPTY": -10, "LAUNCH": -11, "OP": -12,
       "BYTEORDER": -13, "DOMAIN": -14}

KERNELS = ("none", "ew_rows", "ew_tiled", "ew_generic", "red_rows", "red_cols", "red_generic", "ew_interleave")

EXPORTS = ("ocn_unary", "ocn_binary", "ocn_cast_copy", "ocn_reduce", "ocn_reduce_workspace_bytes",
           "ocn_promote", "ocn_dtype_size", "ocn_error_string", "ocn_last_hip_error",
           "ocn_plan_unary", "ocn_plan_binary", "ocn_plan_reduce",
           "ocn_binary_reduce", "ocn_binary_reduce_workspace_bytes", "ocn_plan_binary_reduce",
           "ocn_index_offsets", "ocn_mask_offsets", "ocn_mask_offsets_workspace_bytes", "ocn_gather",
           "ocn_scatter", "ocn_domain_check", "ocn_domain_check_workspace_bytes", "ocn_reduce_scratch",
           "ocn_unary_mode", "ocn_unary_mode_workspace_bytes", "ocn_set_max_launch_blocks")


class OcnTensor(C.Structure):
    _fields_ = [("base", C.c_void_p), ("offset", C.c_int64), ("dtype", C.c_int32),
                ("ndim", C.c_int32), ("size", C.c_int64 * MAX_DIMS),
                ("stride", C.c_int64 * MAX_DIMS), ("device", C.c_int32), ("byteswapped", C.c_int32)]


class OcnPlanInfo(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("compute_dtype", C.c_int32), ("ndim", C.c_int32),
                ("nred", C.c_int32), ("size", C.c_int64 * MAX_DIMS),
                ("stride_out", C.c_int64 * MAX_DIMS), ("stride_a", C.c_int64 * MAX_DIMS),
                ("stride_b", C.c_int64 * MAX_DIMS), ("offset_out", C.c_int64),
                ("offset_a", C.c_int64), ("offset_b", C.c_int64),
                ("red_size", C.c_int64 * MAX_DIMS), ("red_stride_a", C.c_int64 * MAX_DIMS),
                ("vec", C.c_int32), ("tile_log2", C.c_int32 * MAX_DIMS), ("stage_a", C.c_int32),
                ("stage_b", C.c_int32), ("specialised", C.c_int32), ("passes", C.c_int32),
                ("grid", C.c_int64), ("block", C.c_int64), ("split", C.c_int64),
                ("lds_bytes", C.c_int64), ("unclipped", C.c_int64), ("fused", C.c_int64),
                ("tile_group", C.c_int64)]


class OcnError(RuntimeError):
    def __init__(self, code: int):
        msg = lib().ocn_error_string(code).decode()
        if code == ERR["LAUNCH"]:
            msg += f" (hipError {lib().ocn_last_hip_error()})"
        super().__init__(f"ocn error {code}: {msg}")
        self.code = code


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_1810_08723_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_1810_08723_amd.build` (no fallback exists)")
        # PyTorch owns the device memory and the streams the library is handed, so both must run
        # on one HIP runtime: torch is loaded first, and the library then binds to the runtime
        # torch brought (loaded the other way round, the process ends up with two).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        T, I = C.POINTER(OcnTensor), C.POINTER(OcnPlanInfo)
        L.ocn_unary.argtypes = [C.c_int, T, T, C.c_uint32, C.c_void_p]
        L.ocn_binary.argtypes = [C.c_int, T, T, T, C.c_uint32, C.c_void_p]
        L.ocn_cast_copy.argtypes = [T, T, C.c_void_p]
        L.ocn_reduce.argtypes = [C.c_int, T, C.POINTER(C.c_int32), C.c_int32, T, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
        L.ocn_reduce_workspace_bytes.argtypes = [C.c_int, T, C.POINTER(C.c_int32), C.c_int32, T]
        L.ocn_reduce_scratch.argtypes = [C.c_int, T, C.POINTER(C.c_int32), C.c_int32, T, C.c_void_p]
        L.ocn_reduce_workspace_bytes.restype = C.c_size_t
        L.ocn_promote.argtypes = [C.c_int, C.c_int]
        L.ocn_dtype_size.argtypes = [C.c_int]
        L.ocn_error_string.argtypes = [C.c_int]
        L.ocn_error_string.restype = C.c_char_p
        L.ocn_last_hip_error.argtypes = []
        L.ocn_plan_unary.argtypes = [C.c_int, T, T, C.c_uint32, I]
        L.ocn_plan_binary.argtypes = [C.c_int, T, T, T, C.c_uint32, I]
        L.ocn_plan_reduce.argtypes = [C.c_int, T, C.POINTER(C.c_int32), C.c_int32, T, I]
        A = C.POINTER(C.c_int32)
        L.ocn_binary_reduce.argtypes = [C.c_int, C.c_int, T, T, A, C.c_int32, T, C.c_int32, C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.ocn_binary_reduce_workspace_bytes.argtypes = [C.c_int, C.c_int, T, T, A, C.c_int32, T, C.c_int32]
        L.ocn_binary_reduce_workspace_bytes.restype = C.c_size_t
        L.ocn_plan_binary_reduce.argtypes = [C.c_int, C.c_int, T, T, A, C.c_int32, T, C.c_int32, I]
        L.ocn_domain_check_workspace_bytes.argtypes = [C.c_int, T]
        L.ocn_domain_check_workspace_bytes.restype = C.c_size_t
        L.ocn_domain_check.argtypes = [C.c_int, T, T, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ocn_unary_mode_workspace_bytes.argtypes = [C.c_int, C.c_int, T]
        L.ocn_unary_mode_workspace_bytes.restype = C.c_size_t
        L.ocn_unary_mode.argtypes = [C.c_int, C.c_int, T, T, T, C.c_void_p, C.c_size_t, C.POINTER(C.c_int), C.c_void_p]
        L.ocn_set_max_launch_blocks.argtypes = [C.c_int64]
        L.ocn_set_max_launch_blocks.restype = None
        L.ocn_index_offsets.argtypes = [T, C.c_int64, C.c_int64, T, C.c_void_p, C.c_void_p]
        L.ocn_mask_offsets_workspace_bytes.argtypes = [T]
        L.ocn_mask_offsets_workspace_bytes.restype = C.c_size_t
        L.ocn_mask_offsets.argtypes = [T, C.POINTER(C.c_int64), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                       C.c_size_t, C.c_void_p]
        L.ocn_gather.argtypes = [T, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, T, C.c_void_p]
        L.ocn_scatter.argtypes = [T, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, T, C.c_void_p]
        _lib = L
    return _lib


@dataclass
class Tensor:
    """A view on device storage: the descriptor the C ABI takes, plus a keep-alive reference."""
    base: int                      # device address of the storage start
    dtype: str
    sizes: Tuple[int, ...]
    strides: Tuple[int, ...]       # bytes
    offset: int = 0                # bytes
    device: int = 0
    keepalive: Any = field(default=None, repr=False, compare=False)
    byteswapped: bool = False      # the storage holds every scalar in the other byte order

    @staticmethod
    def on_storage(storage, dtype: str, sizes: Sequence[int], strides: Sequence[int],
                   offset: int = 0, byteswapped: bool = False) -> "Tensor":
        """View over a 1-D uint8 torch tensor living on a GPU."""
        dev = storage.device.index if storage.device.index is not None else 0
        return Tensor(storage.data_ptr(), dtype, tuple(sizes), tuple(strides), offset, dev, storage, byteswapped)

    def desc(self) -> OcnTensor:
        # the C struct is rebuilt only when a field has changed (the library never writes to it)
        key = (self.base, self.dtype, self.sizes, self.strides, self.offset, self.device, self.byteswapped)
        cached = self.__dict__.get("_desc_cache")
        if cached is not None and cached[0] == key:
            return cached[1]
        t = OcnTensor()
        t.base = self.base
        t.offset = self.offset
        t.dtype = DTYPE_CODE[self.dtype] if isinstance(self.dtype, str) else int(self.dtype)
        t.ndim = len(self.sizes)
        for d in range(min(len(self.sizes), MAX_DIMS)):
            t.size[d] = self.sizes[d]
            t.stride[d] = self.strides[d]
        t.device = self.device
        t.byteswapped = 1 if self.byteswapped else 0
        self.__dict__["_desc_cache"] = (key, t)
        return t


def _stream(stream) -> int:
    if stream is not None:
        return int(stream)
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _check(rc: int) -> None:
    if rc != OK:
        raise OcnError(rc)


def _scratch(nbytes: int, device: int, stream):
    """A workspace this wrapper allocates on the caller's behalf.  torch's caching allocator ties
    a block to the stream that was current when it was allocated and may hand it out again as
    soon as the last reference is dropped; the kernels that use the block run on `stream`, so
    when that is another stream the block is recorded as in use there and is not reused before
    the enqueued work has finished."""
    import torch
    ws = torch.empty(nbytes, dtype=torch.uint8, device=f"cuda:{device}")
    if stream is not None and int(stream) != int(torch.cuda.current_stream(device).cuda_stream):
        ws.record_stream(torch.cuda.ExternalStream(int(stream), device=f"cuda:{device}"))
    return ws


def _axes(axes: Sequence[int]):
    return (C.c_int32 * max(len(axes), 1))(*axes), len(axes)


def unary(op: str, a: Tensor, out: Tensor, flags: int = 0, stream=None) -> None:
    _check(lib().ocn_unary(UNARY_CODE[op], C.byref(a.desc()), C.byref(out.desc()), flags, _stream(stream)))


def binary(op: str, a: Tensor, b: Tensor, out: Tensor, flags: int = 0, stream=None) -> None:
    _check(lib().ocn_binary(BINARY_CODE[op], C.byref(a.desc()), C.byref(b.desc()),
                            C.byref(out.desc()), flags, _stream(stream)))


def cast_copy(src: Tensor, dst: Tensor, stream=None) -> None:
    _check(lib().ocn_cast_copy(C.byref(src.desc()), C.byref(dst.desc()), _stream(stream)))


def reduce_workspace_bytes(op: str, a: Tensor, axes: Sequence[int], out: Tensor) -> int:
    ax, n = _axes(axes)
    return int(lib().ocn_reduce_workspace_bytes(REDUCE_CODE[op], C.byref(a.desc()), ax, n,
                                                C.byref(out.desc())))


def reduce(op: str, a: Tensor, axes: Sequence[int], out: Tensor, workspace=None, stream=None) -> None:
    """`workspace`: a uint8 torch tensor on the device of at least reduce_workspace_bytes(...)
    bytes, or None to have this wrapper allocate one through torch when the call needs it
    (the library itself never allocates)."""
    ax, n = _axes(axes)
    ws_ptr, ws_bytes = None, 0
    if workspace is None:
        need = reduce_workspace_bytes(op, a, axes, out)
        if need:
            workspace = _scratch(need, a.device, stream)
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel()
    _check(lib().ocn_reduce(REDUCE_CODE[op], C.byref(a.desc()), ax, n, C.byref(out.desc()),
                            ws_ptr, ws_bytes, _stream(stream)))


REDUCE_SCRATCH_BYTES = 1 << 20


def reduce_scratch(op: str, a: Tensor, axes: Sequence[int], out: Tensor, stream=None) -> None:
    """ocn_reduce without a workspace: partial results go to the library's fixed device array
    (at most REDUCE_SCRATCH_BYTES); nothing is allocated, here or in the library."""
    ax, n = _axes(axes)
    _check(lib().ocn_reduce_scratch(REDUCE_CODE[op], C.byref(a.desc()), ax, n, C.byref(out.desc()),
                                    _stream(stream)))


def binary_reduce_workspace_bytes(ew_op: str, red_op: str, a: Tensor, b: Tensor, axes: Sequence[int],
                                  out: Tensor, mid_dtype: str) -> int:
    ax, n = _axes(axes)
    return int(lib().ocn_binary_reduce_workspace_bytes(BINARY_CODE[ew_op], REDUCE_CODE[red_op], C.byref(a.desc()),
                                                       C.byref(b.desc()), ax, n, C.byref(out.desc()),
                                                       DTYPE_CODE[mid_dtype]))


def binary_reduce(ew_op: str, red_op: str, a: Tensor, b: Tensor, axes: Sequence[int], out: Tensor,
                  mid_dtype: str, workspace=None, stream=None) -> None:
    """reduce(red_op, binary(ew_op, a, b) as mid_dtype, axes) -> out; `workspace` as for reduce()."""
    ax, n = _axes(axes)
    ws_ptr, ws_bytes = None, 0
    if workspace is None:
        need = binary_reduce_workspace_bytes(ew_op, red_op, a, b, axes, out, mid_dtype)
        if need:
            workspace = _scratch(need, a.device, stream)
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel()
    _check(lib().ocn_binary_reduce(BINARY_CODE[ew_op], REDUCE_CODE[red_op], C.byref(a.desc()), C.byref(b.desc()),
                                   ax, n, C.byref(out.desc()), DTYPE_CODE[mid_dtype], ws_ptr, ws_bytes,
                                   _stream(stream)))


def index_offsets(index: Tensor, dim_size: int, stride_bytes: int, offsets: Tensor, invalid_count, stream=None) -> None:
    """`invalid_count`: a 1-element int64 torch tensor on the device (overwritten)."""
    _check(lib().ocn_index_offsets(C.byref(index.desc()), dim_size, stride_bytes, C.byref(offsets.desc()),
                                   invalid_count.data_ptr(), _stream(stream)))


def mask_offsets(mask: Tensor, target_strides: Sequence[int], offsets, count, workspace=None, stream=None) -> None:
    """`offsets`: int64 torch tensor on the device (its length is the capacity); `count`: 1-element
    int64 torch tensor; `workspace`: uint8 torch tensor or None to allocate one through torch."""
    need = int(lib().ocn_mask_offsets_workspace_bytes(C.byref(mask.desc())))
    if workspace is None:
        workspace = _scratch(max(need, 8), mask.device, stream)
    ts = (C.c_int64 * max(len(target_strides), 1))(*target_strides)
    _check(lib().ocn_mask_offsets(C.byref(mask.desc()), ts, offsets.data_ptr() if offsets.numel() else None,
                                  offsets.numel(), count.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                  _stream(stream)))


def gather(a_inner: Tensor, offsets, lo: int, hi: int, out: Tensor, stream=None) -> None:
    """`offsets`: int64 torch tensor on the device, one entry per row of `out`."""
    _check(lib().ocn_gather(C.byref(a_inner.desc()), offsets.data_ptr() if offsets.numel() else None,
                            offsets.numel(), lo, hi, C.byref(out.desc()), _stream(stream)))


def scatter(src: Tensor, offsets, lo: int, hi: int, out_inner: Tensor, stream=None) -> None:
    _check(lib().ocn_scatter(C.byref(src.desc()), offsets.data_ptr() if offsets.numel() else None,
                             offsets.numel(), lo, hi, C.byref(out_inner.desc()), _stream(stream)))


def domain_check(op: str, a: Tensor, flag=None, workspace=None, stream=None):
    """Enqueues the domain check of unary `op` over `a` into `flag` (a 1-element bool torch tensor
    on the device; created when None) and returns that tensor without synchronising."""
    import torch
    if flag is None:
        flag = torch.zeros(1, dtype=torch.bool, device=f"cuda:{a.device}")
    tf = Tensor(flag.data_ptr(), "bool", (), (), 0, a.device, flag)
    if workspace is None:
        need = int(lib().ocn_domain_check_workspace_bytes(UNARY_CODE[op], C.byref(a.desc())))
        workspace = _scratch(need, a.device, stream)
    _check(lib().ocn_domain_check(UNARY_CODE[op], C.byref(a.desc()), C.byref(tf.desc()), workspace.data_ptr(),
                                  workspace.numel(), _stream(stream)))
    return flag


MODES = ("standard", "warning", "error", "complex")


def unary_mode(op: str, mode: str, a: Tensor, out: Tensor, out_complex: Optional[Tensor] = None, workspace=None,
               stream=None) -> dict:
    """A unary operation in a compute mode (standard, warning, error, complex).  Returns
    {"outside": None (not checked) | bool, "wrote": "out" | "out_complex"}; error mode raises
    OcnError with code ERR["DOMAIN"] when an element is outside the domain.  `workspace` as for
    reduce()."""
    m = MODES.index(mode)
    need = int(lib().ocn_unary_mode_workspace_bytes(UNARY_CODE[op], m, C.byref(a.desc())))
    ws_ptr, ws_bytes = None, 0
    if workspace is None and need:
        workspace = _scratch(need, a.device, stream)
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel()
    outside = C.c_int(-1)
    oc = C.byref(out_complex.desc()) if out_complex is not None else None
    _check(lib().ocn_unary_mode(UNARY_CODE[op], m, C.byref(a.desc()), C.byref(out.desc()), oc, ws_ptr, ws_bytes,
                                C.byref(outside), _stream(stream)))
    flag = None if outside.value < 0 else bool(outside.value)
    return {"outside": flag, "wrote": "out_complex" if (flag and mode == "complex") else "out"}


def set_max_launch_blocks(blocks: int) -> None:
    """Upper bound on the workgroups of one launch (0: the default, 2^24 - 1)."""
    lib().ocn_set_max_launch_blocks(blocks)


def promote(a: str, b: str) -> str:
    rc = lib().ocn_promote(DTYPE_CODE[a], DTYPE_CODE[b])
    _check(rc if rc < 0 else OK)
    return DTYPES[rc]


def dtype_size(dtype: str) -> int:
    return int(lib().ocn_dtype_size(DTYPE_CODE[dtype]))


def _info_dict(info: OcnPlanInfo) -> dict:
    n, r = info.ndim, info.nred
    return {
        "kernel": KERNELS[info.kernel], "compute_dtype": DTYPES[info.compute_dtype],
        "ndim": n, "size": tuple(info.size[:n]), "stride_out": tuple(info.stride_out[:n]),
        "stride_a": tuple(info.stride_a[:n]), "stride_b": tuple(info.stride_b[:n]),
        "offset_out": info.offset_out, "offset_a": info.offset_a, "offset_b": info.offset_b,
        "red_size": tuple(info.red_size[:r]), "red_stride_a": tuple(info.red_stride_a[:r]),
        "vec": info.vec, "tile_log2": tuple(info.tile_log2[:n]), "stage_a": bool(info.stage_a),
        "stage_b": bool(info.stage_b), "specialised": bool(info.specialised), "passes": info.passes,
        "grid": info.grid, "block": info.block, "split": info.split, "lds_bytes": info.lds_bytes, "unclipped": bool(info.unclipped),
        "fused": bool(info.fused), "tile_group": info.tile_group,
    }


def plan_unary(op: str, a: Tensor, out: Tensor, flags: int = 0) -> dict:
    info = OcnPlanInfo()
    _check(lib().ocn_plan_unary(UNARY_CODE[op], C.byref(a.desc()), C.byref(out.desc()), flags, C.byref(info)))
    return _info_dict(info)


def plan_binary(op: str, a: Tensor, b: Tensor, out: Tensor, flags: int = 0) -> dict:
    info = OcnPlanInfo()
    _check(lib().ocn_plan_binary(BINARY_CODE[op], C.byref(a.desc()), C.byref(b.desc()),
                                 C.byref(out.desc()), flags, C.byref(info)))
    return _info_dict(info)


def plan_binary_reduce(ew_op: str, red_op: str, a: Tensor, b: Tensor, axes: Sequence[int], out: Tensor,
                       mid_dtype: str) -> dict:
    info = OcnPlanInfo()
    ax, n = _axes(axes)
    _check(lib().ocn_plan_binary_reduce(BINARY_CODE[ew_op], REDUCE_CODE[red_op], C.byref(a.desc()),
                                        C.byref(b.desc()), ax, n, C.byref(out.desc()), DTYPE_CODE[mid_dtype],
                                        C.byref(info)))
    return _info_dict(info)


def plan_reduce(op: str, a: Tensor, axes: Sequence[int], out: Tensor) -> dict:
    info = OcnPlanInfo()
    ax, n = _axes(axes)
    _check(lib().ocn_plan_reduce(REDUCE_CODE[op], C.byref(a.desc()), ax, n, C.byref(out.desc()), C.byref(info)))
    return _info_dict(info)
