"""ocn_reduce_scratch (the reduction entry point that allocates nothing: partial results of a
split reduction go to a fixed array inside the library's device image) against ocn_reduce with
a caller-provided workspace: same kernels and launch shapes, so the results must agree bit for
bit - also for floating sums - on calls in a row that share the array, the later ones with
smaller inputs."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def _both(op, x, axes, out_dtype, out_shape):
    """Runs the reduction through both entry points; returns (scratch result, workspace result,
    plan)."""
    import torch
    import paper_1810_08723_amd as ocn
    o1, o2 = View.empty(out_dtype, out_shape), View.empty(out_dtype, out_shape)
    dv = H.DeviceViews()
    tx, t1, t2 = dv.tensor(x), dv.tensor(o1), dv.tensor(o2)
    for v in (o1, o2):
        dv._by_id[id(v.storage)][1].fill_(0x5A)
    plan = ocn.plan_reduce(op, tx, list(axes), t1)
    need = ocn.reduce_workspace_bytes(op, tx, list(axes), t2)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ocn.reduce_scratch(op, tx, list(axes), t1)
    assert torch.cuda.memory_allocated() == before      # nothing came from torch's allocator
    ocn.reduce(op, tx, list(axes), t2, workspace=ws)
    torch.cuda.synchronize()
    return dv.download(o1).copy(), dv.download(o2).copy(), plan, need


def test_scratch_entry_point_matches_the_workspace_entry_point_on_calls_in_a_row():
    from oracle import binding as O
    rng = rng_for(15001)
    # 1. full int8 -> int64 sum (rows kernel, split over workgroups), then a smaller one
    for n in ((1 << 24) + 12345, (1 << 21) + 77):
        x = View.from_numpy(rng.integers(-128, 127, size=n, endpoint=True, dtype=np.int8))
        got, ref, plan, need = _both("sum", x, (0,), "int64", ())
        assert plan["split"] > 1 and plan["passes"] == 2 and 0 < need <= (1 << 20)
        assert np.array_equal(got, ref)
        want = View.empty("int64", ())
        O.reduce("sum", x, [0], want)
        assert np.array_equal(got, want.storage)
    # 2. fp32 column sums (columns kernel, row ranges split), then a smaller one
    for rows, cols in ((8192, 1024), (3001, 517)):
        x = View.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32))
        got, ref, plan, need = _both("sum", x, (0,), "float", (cols,))
        assert plan["kernel"] == "red_cols" and plan["split"] > 1 and 0 < need <= (1 << 20)
        bound = 1e-6 * np.abs(x.to_numpy().astype(np.float64)).sum(axis=0)
        g = got.view(np.float32).astype(np.float64)
        assert np.array_equal(got, ref)
        want = View.empty("float", (cols,))
        O.reduce("sum", x, [0], want)
        assert np.all(np.abs(g - want.storage.view(np.float32)) <= bound)
    # 2b. fp32 full sum over a flat vector (rows kernel split over workgroups), float accumulators
    x = View.from_numpy(rng.standard_normal((1 << 23) + 5).astype(np.float32))
    got, ref, plan, need = _both("sum", x, (0,), "float", ())
    assert plan["split"] > 1
    bound = 1e-6 * np.abs(x.to_numpy().astype(np.float64)).sum()
    want = View.empty("float", ())
    O.reduce("sum", x, [0], want)
    assert np.array_equal(got, ref)
    assert abs(float(got.view(np.float32)[0]) - float(want.storage.view(np.float32)[0])) <= bound
    # 2c. complex128 sums (16-byte partial results) and a bool `any` (1-byte partial results)
    z = rng.standard_normal((1 << 20) + 9) + 1j * rng.standard_normal((1 << 20) + 9)
    x = View.from_numpy(z.astype(np.complex128))
    got, ref, plan, need = _both("sum", x, (0,), "cdouble", ())
    assert plan["split"] > 1
    assert np.array_equal(got, ref)
    flags = np.zeros((1 << 22) + 3, dtype=np.bool_)
    for hit in (False, True):
        flags[-5] = hit
        x = View.from_numpy(flags.copy())
        got, ref, plan, need = _both("any", x, (0,), "bool", ())
        assert plan["split"] > 1 and np.array_equal(got, ref) and bool(got[0]) == hit
    # 3. half max over everything (NaN-free), then a one-pass reduction that needs no scratch
    x = View.from_numpy(rng.standard_normal((1 << 22) + 3).astype(np.float16))
    got, ref, plan, need = _both("max", x, (0,), "half", ())
    assert plan["split"] > 1 and np.array_equal(got, ref)
    x = View.from_numpy(rng.standard_normal((300, 1000)).astype(np.float32))
    got, ref, plan, need = _both("sum", x, (1,), "float", (300,))
    assert need == 0 and np.array_equal(got, ref)


def test_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    import paper_1810_08723_amd as ocn
    from paper_1810_08723_amd import binding as B
    # column sums whose partial results exceed the fixed array: [rows, cols] with many columns
    rows, cols = 1 << 12, 1 << 16
    x = torch.zeros(rows * cols, dtype=torch.uint8, device="cuda:0")
    out = torch.full((cols * 8,), 0x5A, dtype=torch.uint8, device="cuda:0")
    tx = ocn.Tensor.on_storage(x, "int8", (rows, cols), (cols, 1))
    to = ocn.Tensor.on_storage(out, "int64", (cols,), (8,))
    need = ocn.reduce_workspace_bytes("sum", tx, [0], to)
    assert need > B.REDUCE_SCRATCH_BYTES
    with pytest.raises(ocn.OcnError) as e:
        ocn.reduce_scratch("sum", tx, [0], to)
    assert e.value.code == B.ERR["WORKSPACE"]
    torch.cuda.synchronize()
    assert bool((out == 0x5A).all())                    # nothing was launched
