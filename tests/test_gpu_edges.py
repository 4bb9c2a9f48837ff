"""Edge cases on the GPU: in-place operation, zero-sized and scalar operands, eight dimensions,
superimposed views of different types on one storage, and tensors beyond 2^31 elements."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def test_in_place_binary_and_unary():
    rng = rng_for(13000)
    a = random_view(rng, "float", (100, 37))
    b = random_view(rng, "float", (37,))
    H.check_binary("add", a, b, a)                       # A += b: out is the identical view as a
    H.check_unary("neg", a, a)
    t = random_view(rng, "int32", (64, 64))
    bt = random_view(rng, "int32", (64, 64)).permute(1, 0)
    H.check_binary("mul", t, bt, t)                      # in place with a staged (transposed) other operand
    H.check_binary("sub", bt, t, t)                      # out aliases the second input


def test_zero_sized_and_scalar_operands():
    rng = rng_for(13001)
    s = View.from_numpy(np.array(2.5, dtype=np.float32))
    a = random_view(rng, "float", (33, 5))
    H.check_binary("mul", a, s, View.empty("float", (33, 5)))
    H.check_binary("mul", s, s.fresh_copy(), View.empty("float", ()))
    z = View.empty("float", (0, 5))
    H.check_binary("add", z, s, View.empty("float", (0, 5)))
    H.check_unary("ident", View.empty("int8", (3, 0, 2)), View.empty("double", (3, 0, 2)))


def test_eight_dimensions_permuted():
    rng = rng_for(13002)
    a = random_view(rng, "int16", (2, 3, 2, 3, 2, 3, 2, 3))
    perm = (7, 3, 5, 1, 0, 6, 2, 4)
    p = a.permute(*perm)
    H.check_unary("ident", p, View.empty("int16", p.sizes))
    H.check_binary("add", p, random_view(rng, "int16", p.sizes), View.empty("int16", p.sizes, order="F"))


def test_imaginary_part_is_a_real_view_on_complex_storage():
    rng = rng_for(13003)
    z = random_view(rng, "cdouble", (40, 9), specials=False)
    imag = z.reinterpret("double", 8)                    # same sizes and strides, +8 bytes, type double
    real = z.reinterpret("double", 0)
    H.check_unary("ident", imag, View.empty("double", (40, 9)))
    H.check_binary("add", real, imag, View.empty("double", (40, 9)))
    # write through the imaginary view: conj by negating the imaginary parts in place
    H.check_unary("neg", imag, imag)


def test_padded_rows_and_byte_offsets():
    rng = rng_for(13004)
    big = random_view(rng, "float", (50, 40))
    v = big.slice(1, 3, 33, 1)                           # rows of 30 floats with a pitch of 40
    H.check_unary("neg", v, View.empty("float", (50, 30)))
    H.check_binary("add", v, v.fresh_copy(), View.empty("double", (50, 30)))


def test_more_than_2_to_the_31_elements():
    # flat int8 tensor of 2^31 + 2^20 elements: 64-bit vector indices in the rows kernel, 64-bit
    # offsets in the full reduction
    n = (1 << 31) + (1 << 20)
    rng = rng_for(13005)
    x = rng.integers(-128, 127, size=n, endpoint=True, dtype=np.int8)
    a = View.from_numpy(x)
    print("large unary", flush=True)
    H.check_unary("neg", a, View.empty("int8", (n,)))
    print("large reduce", flush=True)
    got, want = H.run_reduce("sum", a, [0], View.empty("int64", ()))
    assert np.array_equal(got, want)


def test_tile_smaller_than_a_batch_of_passes():
    # 256 output elements with a gap between them: one pass of the strided kernel, whose
    # batches hold up to four passes; every element must be written exactly once
    a = View.from_numpy(np.array([2 ** 31 - 1], dtype=np.int32)).broadcast_to((8, 32))
    out = View.empty("double", (8, 63)).slice(1, 0, 63, 2)
    H.check_unary("ident", a, out)
    rng = rng_for(13006)
    b = random_view(rng, "float", (32, 8)).permute(1, 0)
    H.check_binary("add", random_view(rng, "float", (8, 32)), b, View.empty("float", (8, 32)))


def test_diagonal_views():
    # the diagonal of a matrix is a 1-D view whose stride is the sum of the two strides
    rng = rng_for(13010)
    m = random_view(rng, "double", (130, 130), specials=False)
    diag = View(m.storage, "double", (130,), (m.strides[0] + m.strides[1],), m.offset)
    H.check_unary("neg", diag, View.empty("double", (130,)))             # read the diagonal
    ones = View.from_numpy(np.ones((), dtype=np.float64))
    H.check_binary("add", diag, ones, diag)                              # update it in place
    anti = View(m.storage, "double", (130,), (m.strides[0] - m.strides[1],), m.offset + 129 * m.strides[1])
    H.check_binary("mul", diag, anti, View.empty("double", (130,)))     # diagonal times anti-diagonal
    r = View.empty("double", ())
    got, want = H.run_reduce("sum", diag, [0], r)                        # the trace
    assert np.allclose(got.view(np.float64), want.view(np.float64), rtol=1e-13)


@pytest.mark.parametrize("n", (47104, 46500))
def test_transpose_of_more_than_2_to_the_31_elements(n):
    # n x n int8, n*n > 2^31: tile origins need 64 bits, offsets inside a tile stay 32-bit.
    # 47104 = 2^11 * 23 takes the all-vector tiled form, 46500 the general form (clipped tiles).
    # Checked against the definition directly (out[i, j] = x[j, i]) and, on a slab, the oracle.
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    assert n * n > 1 << 31
    rng = rng_for(13100 + n)
    x = rng.integers(-128, 127, size=(n, n), endpoint=True, dtype=np.int8)
    a = View.from_numpy(x).permute(1, 0)
    out = View.empty("int8", (n, n))
    dv = H.DeviceViews()
    plan = ocn.plan_unary("ident", dv.tensor(a), dv.tensor(out))
    assert plan["kernel"] == "ew_tiled" and plan["unclipped"] == (n == 47104), plan
    print("large transpose", n, flush=True)
    ocn.unary("ident", dv.tensor(a), dv.tensor(out))
    torch.cuda.synchronize()
    got = dv.download(out).reshape(n, n).view(np.int8)
    assert np.array_equal(got, x.T)
    # the same through the oracle on a slab of the view (the last 64 rows of the output)
    slab = a.slice(0, n - 64, n, 1)
    want = View.empty("int8", (64, n))
    O.unary("ident", slab, want)
    assert np.array_equal(got[n - 64:], want.to_numpy())
