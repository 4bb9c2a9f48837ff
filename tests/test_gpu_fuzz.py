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
        a = random_strided_view(rng, dt, shape, allow_broadcast=False)
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
