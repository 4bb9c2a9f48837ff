"""First GPU parity checks: one case per kernel family, through the C ABI, against the oracle."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def test_rows_add_float():
    rng = rng_for(101)
    a = random_view(rng, "float", (37, 129))
    b = random_view(rng, "float", (37, 129))
    H.check_binary("add", a, b, View.empty("float", (37, 129)))


def test_rows_broadcast_mixed():
    rng = rng_for(102)
    a = random_view(rng, "int32", (65, 300))
    b = random_view(rng, "float", (1, 300))
    H.check_binary("mul", a, b, View.empty("float", (65, 300)))


def test_cast_flipped_double_to_int16():
    rng = rng_for(103)
    a = random_view(rng, "double", (50, 72)).flip(0)
    H.check_unary("ident", a, View.empty("int16", (50, 72)))


def test_tiled_transpose_add():
    rng = rng_for(104)
    a = random_view(rng, "float", (64, 48, 32), specials=False)
    b = random_view(rng, "float", (32, 64, 48), specials=False).permute(1, 2, 0)
    H.check_binary("add", a, b, View.empty("float", (64, 48, 32)))


def test_tiled_ragged_transpose():
    rng = rng_for(105)
    a = random_view(rng, "double", (70, 45))
    b = random_view(rng, "double", (45, 70)).permute(1, 0)
    H.check_binary("sub", a, b, View.empty("double", (70, 45)))


def test_interp_mixed_types():
    rng = rng_for(106)
    a = random_view(rng, "int16", (9, 33))
    b = random_view(rng, "double", (9, 33))
    H.check_binary("add", a, b, View.empty("half", (9, 33)))
    H.check_binary("lt", a, b, View.empty("int32", (9, 33)))


@pytest.mark.parametrize("axis", [0, 1])
def test_reduce_sum_float(axis):
    rng = rng_for(107)
    x = rng.standard_normal((300, 517)).astype(np.float32)
    a = View.from_numpy(x)
    out = View.empty("float", (517,) if axis == 0 else (300,))
    got, want = H.run_reduce("sum", a, [axis], out)
    g = got.view(np.float32)
    w = want.view(np.float32)
    bound = 1e-6 * np.abs(x.astype(np.float64)).sum(axis=axis)
    assert np.all(np.abs(g.astype(np.float64) - w.astype(np.float64)) <= bound)


def test_reduce_full_int8():
    rng = rng_for(108)
    x = rng.integers(-128, 127, size=1 << 20, endpoint=True).astype(np.int8)
    got, want = H.run_reduce("sum", View.from_numpy(x), [0], View.empty("int64", ()))
    assert np.array_equal(got, want)


def test_reduce_max_half():
    rng = rng_for(109)
    x = rng.standard_normal((200, 1000)).astype(np.float16)
    got, want = H.run_reduce("max", View.from_numpy(x), [1], View.empty("half", (200,)))
    assert np.array_equal(got, want)
