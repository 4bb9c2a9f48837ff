"""The five benchmark configurations as seeded synthetic inputs.

Each case is one call of the engine: operand views, the operation, the output view, the
logical byte count (distinct input elements read + output elements written, broadcast
operands counted once) and how results are compared.  The paper has no datasets; these
tensors restate the configurations the build is measured on, "contiguous" read row-major.

Seeds: PCG64(1810087230 + 10 * config + tensor_index); normals are drawn in float64 and
rounded to the tensor dtype; NaNs of configuration 2 are planted where a uniform draw from the
same generator, taken after the values, falls below 1e-4.

Only random draws and view construction live here - none of the engine's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .values import rng_for
from .views import View, itemsize

BASE_SEED = 1810087230


@dataclass
class Case:
    name: str
    kind: str                      # "binary" | "unary" | "reduce" | "binary_reduce"
    op: str
    inputs: List[View]
    out: View
    axes: Tuple[int, ...] = ()
    logical_bytes: int = 0
    compare: str = "exact"         # "exact" | "sum" (bounded error relative to sum |x|) | "ulp" (rel_bound units
                                   # in the last place of the oracle value; complex: of its magnitude)
    rel_bound: float = 0.0         # for compare == "sum"
    note: str = ""
    red_op: str = ""               # kind == "binary_reduce": reduce(red_op, binary(op, a, b) as mid_dtype, axes)
    mid_dtype: str = ""


def _seed(config: int, tensor: int) -> int:
    return BASE_SEED + 10 * config + tensor


def _uniform_pm1(seed: int, sizes) -> np.ndarray:
    return (rng_for(seed).random(sizes, dtype=np.float32) * np.float32(2) - np.float32(1)).astype(np.float32)


def _normal(seed: int, sizes, dtype, sigma: float = 1.0) -> np.ndarray:
    x = rng_for(seed).standard_normal(sizes)
    if sigma != 1.0:
        x *= sigma
    return x.astype(dtype)


def config1(scale: int = 1) -> Case:
    """fp32 add C = A + B; A, C contiguous [64,48,32]*scale; B a contiguous [32,64,48]*scale
    buffer read with dims permuted (1,2,0)."""
    n0, n1, n2 = 64 * scale, 48 * scale, 32 * scale
    a = View.from_numpy(_uniform_pm1(_seed(0, 0), (n0, n1, n2)))
    b = View.from_numpy(_uniform_pm1(_seed(0, 1), (n2, n0, n1))).permute(1, 2, 0)
    out = View.empty("float", (n0, n1, n2))
    n = n0 * n1 * n2
    return Case("C1" if scale == 1 else f"C1x{scale}", "binary", "add", [a, b], out,
                logical_bytes=12 * n, note="transposed second operand")


def config2(rows: int = 4096, cols: int = 4096) -> Case:
    """fp64 -> int16 cast-copy of a [rows, cols] input with rows flipped; N(0, sigma=2e4),
    NaN at rate 1e-4."""
    rng = rng_for(_seed(1, 0))
    x = rng.standard_normal((rows, cols))
    x *= 2e4
    x[rng.random((rows, cols)) < 1e-4] = np.nan
    src = View.from_numpy(x).flip(0)
    out = View.empty("int16", (rows, cols))
    return Case("C2", "unary", "ident", [src], out, logical_bytes=10 * rows * cols,
                note="negative stride on axis 0")


def config3(rows: int = 8192, cols: int = 8192) -> Case:
    """C = A * B; A int32 [rows, cols] uniform in [-1000, 1000]; B float32 [1, cols] with stride
    0 on axis 0, N(0,1); C float32."""
    a = rng_for(_seed(2, 0)).integers(-1000, 1000, size=(rows, cols), endpoint=True, dtype=np.int64).astype(np.int32)
    b = _normal(_seed(2, 1), (1, cols), np.float32)
    va = View.from_numpy(a)
    vb = View.from_numpy(b).broadcast_to((rows, cols))
    out = View.empty("float", (rows, cols))
    return Case("C3", "binary", "mul", [va, vb], out, logical_bytes=8 * rows * cols + 4 * cols,
                note="broadcast row, int32 promoted on load")


def config4(rows: int = 16384, cols: int = 4096, n_full: int = 1 << 28) -> List[Case]:
    """Reductions: fp32 sum over axis 1 and axis 0 of [rows, cols] N(0,1); fp16 max over axis 1 of
    the same shape; full int8 -> int64 sum over n_full elements uniform in [-128, 127]."""
    x32 = _normal(_seed(3, 0), (rows, cols), np.float32)
    v32 = View.from_numpy(x32)
    x16 = _normal(_seed(3, 1), (rows, cols), np.float16)
    v16 = View.from_numpy(x16)
    x8 = rng_for(_seed(3, 2)).integers(-128, 127, size=n_full, endpoint=True, dtype=np.int8)
    v8 = View.from_numpy(x8)
    n = rows * cols
    return [
        Case("C4a", "reduce", "sum", [v32], View.empty("float", (rows,)), axes=(1,),
             logical_bytes=4 * n + 4 * rows, compare="sum", rel_bound=1e-6, note="reduced axis fastest"),
        Case("C4b", "reduce", "sum", [v32], View.empty("float", (cols,)), axes=(0,),
             logical_bytes=4 * n + 4 * cols, compare="sum", rel_bound=1e-6, note="kept axis fastest"),
        Case("C4c", "reduce", "max", [v16], View.empty("half", (rows,)), axes=(1,),
             logical_bytes=2 * n + 2 * rows, note="half precision max"),
        Case("C4d", "reduce", "sum", [v8], View.empty("int64", ()), axes=(0,),
             logical_bytes=n_full + 8, note="full two-pass reduction"),
    ]


def config5(shape: Sequence[int] = (16, 32, 64, 64, 8), reading: str = "R1") -> List[Case]:
    """complex64 multiply on logical shape [16,32,64,64,8]: A is a step-2 slice along axis 2 of a
    permuted buffer (4,2,0,3,1); B contiguous; C written permuted (3,0,4,1,2).  Also the bool
    mask |A| > |B| (contiguous).

    The layout sentence admits two readings, both built here:
      R1  view.dim[i] = buffer.dim[perm[i]] (the convention of configuration 1);
      R2  the buffer stores the logical dims in the order perm (slowest first).
    They are two stride vectors for the same operation; R2's cases are named C5b / C5bm."""
    s0, s1, s2, s3, s4 = shape
    a_logical = (s0, s1, 2 * s2, s3, s4)   # before the step-2 slice
    perm_a, perm_c = (4, 2, 0, 3, 1), (3, 0, 4, 1, 2)

    def cplx(seed, sizes):
        rng = rng_for(seed)
        z = np.empty(sizes, dtype=np.complex64)
        z.real = rng.standard_normal(sizes).astype(np.float32)
        z.imag = rng.standard_normal(sizes).astype(np.float32)
        return z

    if reading == "R1":
        pa_shape = [0] * 5
        for i, p in enumerate(perm_a):
            pa_shape[p] = a_logical[i]
        pc_shape = [0] * 5
        for i, p in enumerate(perm_c):
            pc_shape[p] = shape[i]
        view_perm_a, view_perm_c = perm_a, perm_c
        suffix = ""
    elif reading == "R2":
        pa_shape = [a_logical[p] for p in perm_a]
        pc_shape = [shape[p] for p in perm_c]
        # logical dim i sits at buffer axis perm.index(i)
        view_perm_a = tuple(perm_a.index(i) for i in range(5))
        view_perm_c = tuple(perm_c.index(i) for i in range(5))
        suffix = "b"
    else:
        raise ValueError(reading)

    pa = View.from_numpy(cplx(_seed(4, 0), tuple(pa_shape)))
    a = pa.permute(*view_perm_a).slice(2, 0, 2 * s2, 2)
    b = View.from_numpy(cplx(_seed(4, 1), tuple(shape)))
    pc = View.empty("cfloat", tuple(pc_shape))
    c = pc.permute(*view_perm_c)
    assert a.sizes == tuple(shape) and c.sizes == tuple(shape)
    n = int(np.prod(shape))
    mask = View.empty("bool", tuple(shape))
    return [
        Case("C5" + suffix, "binary", "mul", [a, b], c, logical_bytes=24 * n,
             note="three different fastest axes"),
        Case("C5" + suffix + "m", "binary", "absgt", [a, b], mask, logical_bytes=17 * n,
             note="bool mask |A|>|B|"),
    ]


def fused_cases(rows: int = 16384, cols: int = 4096, n_flat: int = 1 << 26) -> List[Case]:
    """Reductions of an elementwise result (the step after the five configurations): row-wise
    and column-wise inner products of two fp32 [rows, cols] matrices N(0,1), and the count of
    a > b over two flat fp32 vectors.  Logical bytes: both inputs once plus the output."""
    a = View.from_numpy(_normal(_seed(5, 0), (rows, cols), np.float32))
    b = View.from_numpy(_normal(_seed(5, 1), (rows, cols), np.float32))
    x = View.from_numpy(_normal(_seed(5, 2), (n_flat,), np.float32))
    y = View.from_numpy(_normal(_seed(5, 3), (n_flat,), np.float32))
    return [
        Case("F1", "binary_reduce", "mul", [a, b], View.empty("float", (rows,)), axes=(1,),
             logical_bytes=8 * rows * cols + 4 * rows, compare="sum", rel_bound=1e-6,
             note="row-wise inner products", red_op="sum", mid_dtype="float"),
        Case("F2", "binary_reduce", "gt", [x, y], View.empty("int64", ()), axes=(0,),
             logical_bytes=8 * n_flat + 8, note="count of a > b", red_op="sum", mid_dtype="bool"),
        Case("F3", "binary_reduce", "mul", [a, b], View.empty("float", (cols,)), axes=(0,),
             logical_bytes=8 * rows * cols + 4 * cols, compare="sum", rel_bound=1e-6,
             note="column-wise inner products", red_op="sum", mid_dtype="float"),
    ]


def elementary_cases(n_flat: int = 1 << 26, n_cplx: int = 1 << 24) -> List[Case]:
    """Elementary functions: exp over a flat fp32 vector uniform in [-9, 9), sin over a complex64
    vector with parts uniform in [-5, 5).  Compared within a few units in the last place."""
    x = (rng_for(_seed(6, 0)).random(n_flat, dtype=np.float32) * np.float32(18) - np.float32(9)).astype(np.float32)
    rng = rng_for(_seed(6, 1))
    z = np.empty(n_cplx, dtype=np.complex64)
    z.real = rng.random(n_cplx, dtype=np.float32) * np.float32(10) - np.float32(5)
    z.imag = rng.random(n_cplx, dtype=np.float32) * np.float32(10) - np.float32(5)
    return [
        Case("E1", "unary", "exp", [View.from_numpy(x)], View.empty("float", (n_flat,)),
             logical_bytes=8 * n_flat, compare="ulp", rel_bound=4, note="exp, fp32"),
        Case("E2", "unary", "sin", [View.from_numpy(z)], View.empty("cfloat", (n_cplx,)),
             logical_bytes=16 * n_cplx, compare="ulp", rel_bound=8, note="complex sine"),
    ]


def layout_cases(scale: int = 1) -> List[Case]:
    """Shapes and types outside the five configurations, measured beside them: a transpose with
    extents that are not powers of two, a channel-first to channel-last copy with three channels
    (an output whose fastest axis is 12 bytes long), an operation on a combination of types that
    has no kernel of its own, the full sum of an every-other-element view, and the contiguous
    cast and the row sums of configurations 2 and 4 on operands stored in the other byte order.
    `scale` > 1 shrinks every case for tests."""
    def sz(n):
        return max(n // scale, 8)
    n0, n1 = sz(6000), sz(5000)
    a = View.from_numpy(_uniform_pm1(_seed(7, 0), (n0, n1)))
    b = View.from_numpy(_uniform_pm1(_seed(7, 1), (n1, n0))).permute(1, 0)
    nb, hw = sz(64), sz(512)
    img = View.from_numpy(_uniform_pm1(_seed(7, 2), (nb, 3, hw, hw)))
    ne = sz(1 << 25)
    i16 = View.from_numpy(rng_for(_seed(7, 3)).integers(-30000, 30000, size=ne).astype(np.int16))
    f32 = View.from_numpy(_uniform_pm1(_seed(7, 4), (ne,)))
    ns = sz(1 << 27)
    strided = View.from_numpy(_normal(_seed(7, 5), (ns,), np.float32)).slice(0, 0, ns, 2)
    rows2, cols2 = sz(4096), sz(4096)
    x64 = rng_for(_seed(7, 6)).standard_normal((rows2, cols2))
    x64 *= 2e4
    swapped64 = View.from_numpy(x64).in_other_byte_order().flip(0)
    r4, c4 = sz(16384), sz(4096)
    swapped32 = View.from_numpy(_normal(_seed(7, 7), (r4, c4), np.float32)).in_other_byte_order()
    return [
        Case("L1", "binary", "add", [a, b], View.empty("float", (n0, n1)), logical_bytes=12 * n0 * n1,
             note="transpose, extents not powers of two (general tiled form)"),
        Case("L2", "unary", "ident", [img.permute(0, 2, 3, 1)], View.empty("float", (nb, hw, hw, 3)),
             logical_bytes=8 * nb * 3 * hw * hw, note="channel-first to channel-last, 3 channels"),
        Case("L3", "binary", "add", [i16, f32], View.empty("double", (ne,)), logical_bytes=14 * ne,
             note="int16 + float -> double: no kernel of its own (generic-dtype kernel)"),
        Case("L4", "reduce", "sum", [strided], View.empty("float", ()), axes=(0,), logical_bytes=4 * (ns // 2) + 4,
             compare="sum", rel_bound=1e-6, note="full sum of an every-other-element view"),
        Case("S2", "unary", "ident", [swapped64], View.empty("int16", (rows2, cols2)), logical_bytes=10 * rows2 * cols2,
             note="configuration 2 with the input in the other byte order"),
        Case("S4", "reduce", "sum", [swapped32], View.empty("float", (r4,)), axes=(1,), logical_bytes=4 * r4 * c4 + 4 * r4,
             compare="sum", rel_bound=1e-6, note="configuration 4 (sum over axis 1) with the input in the other byte order"),
    ]


def all_cases_full() -> List[Case]:
    """Every benchmark case at full size (about 3.2 GB of host memory).  The multiply and the mask
    of configuration 5 read the same A and B; the two readings are interleaved so that neither
    runs directly after the case that shares its inputs (it would find part of them cached)."""
    mul, mask = config5()
    mul_b, mask_b = config5(reading="R2")
    return [config1(1), config1(8), config2(), config3(), *config4(), mul, mul_b, mask, mask_b]


def all_cases_small() -> List[Case]:
    """The same cases shrunk so the CPU oracle finishes in seconds; still several tiles and a
    ragged tail in every kernel."""
    return [config1(1), config1(2), config2(301, 517), config3(263, 1031),
            *config4(389, 1021, (1 << 20) + 77), *config5((6, 10, 12, 18, 8)),
            *config5((6, 10, 12, 18, 8), reading="R2")]
