"""GPU parity of the full 15 x 15 cast matrix (ocn_cast_copy) on strided, reversed and permuted
views with special values, through every elementwise kernel family.  Bit-exact."""
import itertools

import numpy as np
import pytest

import exactmath as X
import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("src", X.ALL)
def test_cast_matrix_rows_kernel(src):
    # contiguous rows with a reversed outer axis and a ragged tail: the vectorised rows kernel
    rng = rng_for(8000 + X.ALL.index(src))
    a = random_view(rng, src, (37, 203)).flip(0)
    for dst in X.ALL:
        print("cast", src, "->", dst, flush=True)
        H.check_unary("ident", a, View.empty(dst, (37, 203)))


@pytest.mark.parametrize("src", X.ALL)
def test_cast_matrix_tiled_kernel(src):
    # transposed source: staged through LDS
    rng = rng_for(8100 + X.ALL.index(src))
    a = random_view(rng, src, (70, 45)).permute(1, 0)
    for dst in X.ALL:
        print("cast/T", src, "->", dst, flush=True)
        H.check_unary("ident", a, View.empty(dst, (45, 70)))


@pytest.mark.parametrize("src", X.ALL)
def test_cast_matrix_strided_output(src):
    # output with a gap between elements: plain strided kernel, untouched bytes must survive
    rng = rng_for(8200 + X.ALL.index(src))
    a = random_view(rng, src, (19, 31))
    for dst in X.ALL:
        out = View.empty(dst, (19, 62)).slice(1, 1, 62, 2)
        H.check_unary("ident", a, out)


def test_config2_edge_values_on_gpu():
    x = np.array([1.9, -1.9, 32767.4, 32767.9, 32768.0, 4e4, -32768.9, -32769.0, -4e4, np.nan, 0.5, -0.5,
                  np.inf, -np.inf, 1e300, -1e300, 5e-324, -0.0] * 7)
    H.check_unary("ident", View.from_numpy(x), View.empty("int16", x.shape))


def test_double_to_half_rounds_once():
    # values where rounding double -> float -> half would differ from rounding double -> half
    base = np.float64(np.float16(1.0)) + 2.0 ** -11          # exactly between two halfs
    xs = np.array([base + 2.0 ** -30, base - 2.0 ** -30, base, -base - 2.0 ** -40, 65519.999999, 65520.0,
                   2.0 ** -25 + 2.0 ** -60, 2.0 ** -25, 6.1e-5, 5.96e-8, 1e-9] * 9)
    H.check_unary("ident", View.from_numpy(xs), View.empty("half", xs.shape))
    rng = rng_for(8300)
    r = np.ldexp(rng.standard_normal(20000), rng.integers(-28, 18, size=20000))
    H.check_unary("ident", View.from_numpy(r), View.empty("half", r.shape))
    H.check_unary("ident", View.from_numpy(r), View.empty("chalf", r.shape))


def test_wide_integers_to_floating_types():
    rng = rng_for(8301)
    i64 = rng.integers(-2 ** 63, 2 ** 63 - 1, size=30000, dtype=np.int64, endpoint=True)
    u64 = rng.integers(0, 2 ** 64, size=30000, dtype=np.uint64)
    for dst in ("half", "float", "double", "cfloat"):
        H.check_unary("ident", View.from_numpy(i64), View.empty(dst, i64.shape))
        H.check_unary("ident", View.from_numpy(u64), View.empty(dst, u64.shape))
    near = (np.int64(1) << np.arange(20, 63)).repeat(6) + np.tile(np.array([-2, -1, 0, 1, 2, 3]), 43)
    H.check_unary("ident", View.from_numpy(near), View.empty("float", near.shape))
