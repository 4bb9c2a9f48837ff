"""GPU parity on the five benchmark configurations, reduced and full size, through the C ABI,
in the launch configuration the benchmark times.  Bit-exact for integer, bool, cast and IEEE
elementwise results; float sums within 1e-6 * sum|x| (fp32 against the fp64-accumulating
oracle)."""
import numpy as np
import pytest

import gpu_harness as H
from workloads import configs

pytestmark = pytest.mark.gpu

_FLOAT = {"half": np.float16, "float": np.float32, "double": np.float64}


def _run_case(c):
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    dv = H.DeviceViews()
    ins = [dv.tensor(v) for v in c.inputs]
    out = dv.tensor(c.out)
    if c.kind == "binary":
        ocn.binary(c.op, ins[0], ins[1], out)
        dv.torch.cuda.synchronize()
        got = dv.download(c.out)
        O.binary(c.op, c.inputs[0], c.inputs[1], c.out)
    elif c.kind == "unary":
        ocn.unary(c.op, ins[0], out)
        dv.torch.cuda.synchronize()
        got = dv.download(c.out)
        O.unary(c.op, c.inputs[0], c.out)
    elif c.kind == "binary_reduce":
        ocn.binary_reduce(c.op, c.red_op, ins[0], ins[1], list(c.axes), out, c.mid_dtype)
        dv.torch.cuda.synchronize()
        got = dv.download(c.out)
        O.binary_reduce(c.op, c.red_op, c.inputs[0], c.inputs[1], list(c.axes), c.out, c.mid_dtype)
    else:
        ocn.reduce(c.op, ins[0], list(c.axes), out)
        dv.torch.cuda.synchronize()
        got = dv.download(c.out)
        O.reduce(c.op, c.inputs[0], list(c.axes), c.out)
    want = c.out.storage
    if c.compare == "exact":
        assert H.storages_equal(c.out.dtype, got, want), c.name + ": " + H.first_mismatch(c.out.dtype, got, want)
    elif c.compare == "ulp":
        # elementary functions: within rel_bound units in the last place of the oracle value
        cplx = c.out.dtype == "cfloat"
        g = got.view(np.complex64 if cplx else np.float32)
        w = want.view(np.complex64 if cplx else np.float32)
        mag = np.abs(w).astype(np.float32)
        ulp = np.spacing(mag).astype(np.float64)
        for part in ((np.real, np.imag) if cplx else (np.asarray,)):
            err = np.abs(part(g).astype(np.float64) - part(w).astype(np.float64))
            assert np.all(err <= c.rel_bound * ulp), (c.name, float((err / ulp).max()))
    else:
        # |gpu - oracle| <= rel_bound * sum|x| per output
        ft = _FLOAT[c.out.dtype]
        g = got.view(ft).astype(np.float64)
        w = want.view(ft).astype(np.float64)
        x = c.inputs[0].to_numpy().astype(np.float64)
        if c.kind == "binary_reduce":       # the addends are the elementwise results (products here)
            assert c.op == "mul"
            x = x * c.inputs[1].to_numpy().astype(np.float64)
        bound = c.rel_bound * np.abs(x).sum(axis=c.axes)
        err = np.abs(g - w)
        assert np.all(err <= bound.reshape(-1)), (c.name, float(err.max()), float(bound.min()))
        # and the two agree far better than the bound requires (both accumulate in fp64)
        assert np.all(err <= 1e-7 * np.abs(x).sum(axis=c.axes).reshape(-1) + 1e-30)


@pytest.mark.parametrize("idx", range(15))
def test_small_cases(idx):
    c = (configs.all_cases_small() + configs.fused_cases(389, 1021, (1 << 20) + 77))[idx]
    print("case", c.name, c.op, [v.sizes for v in c.inputs], flush=True)
    _run_case(c)


@pytest.mark.parametrize("which", ["C1", "C1x8", "C2", "C3", "C4", "C5", "C5b", "F", "E"])
def test_full_size_cases(which):
    if which == "C1":
        cases = [configs.config1(1)]
    elif which == "C1x8":
        cases = [configs.config1(8)]
    elif which == "C2":
        cases = [configs.config2()]
    elif which == "C3":
        cases = [configs.config3()]
    elif which == "C4":
        cases = configs.config4()
    elif which == "C5":
        cases = configs.config5()
    elif which == "C5b":
        cases = configs.config5(reading="R2")
    elif which == "F":
        cases = configs.fused_cases()
    else:
        cases = configs.elementary_cases()
    for c in cases:
        print("case", c.name, c.op, [v.sizes for v in c.inputs], flush=True)
        _run_case(c)
