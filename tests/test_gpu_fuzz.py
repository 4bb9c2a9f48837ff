"""Randomised descriptors: ranks 0..8, sizes including 0 and 1, permuted / stepped / reversed /
broadcast / offset views, random operations and dtypes.  Bit-exact against the oracle."""
import numpy as np
import pytest

import exactmath as X
import gpu_harness as H
from workloads.fuzz import random_shape, random_strided_view
from workloads.values import rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu

SPECIALISED_T = ("uint8", "int16", "int32", "int64", "half", "float", "double", "cfloat", "cdouble", "bool")


@pytest.mark.parametrize("seed", range(40))
def test_fuzz_elementwise(seed):
    rng = rng_for(11000 + seed)
    for it in range(12):
        shape = random_shape(rng, max_ndim=8 if it % 3 == 0 else 5, max_elems=20000)
        kind = int(rng.integers(0, 4))
        if kind == 0:       # homogeneous arithmetic (specialised kernels)
            T = SPECIALISED_T[int(rng.integers(0, len(SPECIALISED_T)))]
            ops = [o for o in X.ARITH + X.BITWISE if X.binary_supported(o, T)]
            if not ops:
                continue
            op = ops[int(rng.integers(0, len(ops)))]
            da = db = dout = T
        elif kind == 1:     # comparison
            T = SPECIALISED_T[int(rng.integers(0, len(SPECIALISED_T)))]
            ops = [o for o in X.COMPARE if X.binary_supported(o, T)]
            op = ops[int(rng.integers(0, len(ops)))]
            da = db = T
            dout = "bool"
        elif kind == 2:     # cast
            op = None
            da = X.ALL[int(rng.integers(0, 15))]
            dout = X.ALL[int(rng.integers(0, 15))]
        else:               # arbitrary mix (generic-dtype kernel)
            da, db, dout = (X.ALL[int(rng.integers(0, 15))] for _ in range(3))
            ops = [o for o in X.ARITH + X.BITWISE + X.COMPARE + X.LOGICAL
                   if X.binary_supported(o, X.compute_type(o, da, db, dout))]
            op = ops[int(rng.integers(0, len(ops)))]
        a = random_strided_view(rng, da, shape)
        out = random_strided_view(rng, dout, shape, writable=True)
        print("fuzz", seed, it, shape, op, da, dout, a.strides, out.strides, flush=True)
        if op is None:
            H.check_unary("ident", a, out)
        else:
            b = random_strided_view(rng, db, shape)
            H.check_binary(op, a, b, out)


@pytest.mark.parametrize("seed", range(20))
def test_fuzz_reduce(seed):
    rng = rng_for(12000 + seed)
    for it in range(10):
        shape = random_shape(rng, max_ndim=6, max_elems=40000)
        if len(shape) == 0:
            continue
        dt = ("int8", "uint8", "int16", "int32", "int64", "uint32", "bool")[int(rng.integers(0, 7))]
        a = random_strided_view(rng, dt, shape, allow_broadcast=bool(it % 2))   # every other case may have zero strides
        if tuple(a.sizes) != tuple(shape):  # axes left to be broadcast: a reduction wants them spelled out (zero strides)
            while a.ndim < len(shape):
                a = a.unsqueeze(0)
            a = a.broadcast_to(shape)
        naxes = int(rng.integers(0, len(shape) + 1))
        axes = [int(x) for x in rng.permutation(len(shape))[:naxes]]
        kept = [s for d, s in enumerate(shape) if d not in axes]
        op = ("sum", "min", "max", "any", "all")[int(rng.integers(0, 5))]
        nred = int(np.prod([shape[d] for d in axes])) if axes else 1
        if op in ("min", "max") and nred == 0 and int(np.prod(kept)) > 0:
            continue
        out_dt = {"sum": "uint64" if dt.startswith("u") else "int64", "min": dt, "max": dt, "any": "bool", "all": "bool"}[op]
        out = random_strided_view(rng, out_dt, kept, writable=True)
        print("fuzz-reduce", seed, it, shape, axes, op, dt, a.strides, flush=True)
        got, want = H.run_reduce(op, a, axes, out)
        assert np.array_equal(got, want), H.first_mismatch(out_dt, got, want)


def _permuted(rng, dtype, shape, step_axis=None, writable=False):
    """A view of `shape` over a dense buffer whose axes are stored in a random order (and with a
    step of 2 along one axis when asked): positive strides only, power-of-two friendly."""
    from workloads.values import random_view
    nd = len(shape)
    perm = [int(x) for x in rng.permutation(nd)]
    phys = [shape[p] * (2 if p == step_axis else 1) for p in perm]
    base = View.empty(dtype, phys) if writable else random_view(rng, dtype, phys)
    inv = [perm.index(i) for i in range(nd)]
    v = base.permute(*inv)
    if step_axis is not None:
        v = v.slice(step_axis, 0, 2 * shape[step_axis], 2)
    assert v.sizes == tuple(shape)
    return v


@pytest.mark.parametrize("seed", range(24))
def test_fuzz_unclipped_tiles(seed):
    """Power-of-two extents with permuted storage orders: the shapes for which no tile is
    clipped, so the lean all-vector form of the tiled kernel runs (mixed element sizes, one or
    two staged inputs, stepped inputs)."""
    import paper_1810_08723_amd as ocn
    rng = rng_for(11500 + seed)
    combos = [("add", "float", "float", "float"), ("mul", "cfloat", "cfloat", "cfloat"),
              ("absgt", "cfloat", "cfloat", "bool"), ("sub", "int16", "int16", "int16"),
              ("lt", "double", "double", "bool"), ("max", "uint8", "uint8", "uint8"),
              ("mul", "int32", "float", "float"), ("add", "int64", "int64", "int64"),
              (None, "double", None, "int16"), (None, "half", None, "float"), (None, "cdouble", None, "cfloat")]
    for it in range(6):
        nd = int(rng.integers(2, 6))
        shape = [1 << int(rng.integers(1, 7)) for _ in range(nd)]
        while int(np.prod(shape)) > (1 << 17):
            shape[int(rng.integers(0, nd))] = 2
        op, da, db, dout = combos[int(rng.integers(0, len(combos)))]
        step = int(rng.integers(0, nd)) if rng.random() < 0.3 else None
        a = _permuted(rng, da, shape, step_axis=step)
        out = _permuted(rng, dout, shape, writable=True)
        dv = H.DeviceViews()
        if op is None:
            plan = ocn.plan_unary("ident", dv.tensor(a), dv.tensor(out))
        else:
            b = _permuted(rng, db, shape)
            plan = ocn.plan_binary(op, dv.tensor(a), dv.tensor(b), dv.tensor(out))
        print("unclipped fuzz", seed, it, shape, op, da, dout, a.strides, out.strides, plan["kernel"],
              plan["unclipped"], flush=True)
        if op is None:
            H.check_unary("ident", a, out)
        else:
            H.check_binary(op, a, b, out)


@pytest.mark.parametrize("case", range(8))
def test_unclipped_form_on_known_shapes(case):
    """Shapes chosen so that the lean form certainly runs (asserted through the plan)."""
    import paper_1810_08723_amd as ocn
    rng = rng_for(11600 + case)
    from workloads.values import random_view
    spec = [
        ("add", "float", "float", "float", (64, 96, 64), (2, 0, 1), (0, 1, 2), (0, 1, 2)),       # b transposed
        ("mul", "cfloat", "cfloat", "cfloat", (16, 32, 16, 32), (3, 1, 0, 2), (0, 1, 2, 3), (2, 0, 3, 1)),  # three orders
        ("absgt", "cfloat", "cfloat", "bool", (32, 64, 64), (2, 1, 0), (0, 1, 2), (0, 1, 2)),    # mixed sizes
        (None, "double", None, "int16", (256, 128), (1, 0), None, (0, 1)),                        # transposing cast
        ("max", "uint8", "uint8", "uint8", (256, 512), (1, 0), (0, 1), (0, 1)),                   # 16-element vectors
        ("sub", "int16", "int16", "int16", (128, 64, 8), (1, 2, 0), (2, 0, 1), (0, 1, 2)),
        ("lt", "double", "double", "bool", (64, 256), (1, 0), (0, 1), (0, 1)),                    # 8-byte in, 1-byte out
        ("add", "int64", "int64", "int64", (8, 16, 32, 16), (0, 1, 2, 3), (3, 2, 1, 0), (1, 0, 3, 2)),
    ][case]
    op, da, db, dout, shape, pa, pb, po = spec

    def view(dtype, perm, writable=False):
        phys = [shape[p] for p in perm]
        base = View.empty(dtype, phys) if writable else random_view(rng, dtype, phys)
        return base.permute(*[perm.index(i) for i in range(len(shape))])
    a = view(da, pa)
    out = view(dout, po, writable=True)
    dv = H.DeviceViews()
    if op is None:
        plan = ocn.plan_unary("ident", dv.tensor(a), dv.tensor(out))
        assert plan["kernel"] == "ew_tiled" and plan["unclipped"], plan
        H.check_unary("ident", a, out)
    else:
        b = view(db, pb)
        plan = ocn.plan_binary(op, dv.tensor(a), dv.tensor(b), dv.tensor(out))
        assert plan["kernel"] == "ew_tiled" and plan["unclipped"], plan
        H.check_binary(op, a, b, out)


MIXED_PAIRS = [("int32", "float", "float"), ("float", "int32", "float"), ("half", "float", "float"),
               ("float", "half", "float"), ("float", "double", "double"), ("double", "float", "double"),
               ("int32", "double", "double"), ("double", "int32", "double"), ("int64", "double", "double"),
               ("double", "int64", "double"), ("float", "cfloat", "cfloat"), ("cfloat", "float", "cfloat"),
               ("double", "cdouble", "cdouble"), ("cdouble", "double", "cdouble")]


@pytest.mark.parametrize("seed", range(8))
def test_fuzz_mixed_types_converted_on_load(seed):
    """+, -, *, / on the mixed input type pairs that have kernels of their own, over random
    shapes (every third one with power-of-two extents) and random strided views."""
    rng = rng_for(11800 + seed)
    for it in range(10):
        da, db, dout = MIXED_PAIRS[int(rng.integers(0, len(MIXED_PAIRS)))]
        op = ("add", "sub", "mul", "div")[int(rng.integers(0, 4))]
        shape = random_shape(rng, max_ndim=5, max_elems=20000)
        if it % 3 == 0:
            shape = tuple(1 << int(rng.integers(1, 6)) for _ in range(int(rng.integers(2, 5))))
        a = random_strided_view(rng, da, shape)
        b = random_strided_view(rng, db, shape)
        out = random_strided_view(rng, dout, shape, writable=True)
        print("fuzz-mixed", seed, it, op, da, db, shape, a.strides, b.strides, out.strides, flush=True)
        H.check_binary(op, a, b, out)
