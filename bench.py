"""Benchmark: effective GB/s (logical bytes moved) of the strided tensor engine on one MI355X.

One "step" runs every benchmark operation once, through the C ABI, on synthetic inputs that are
already resident in HBM: the five configurations (C1, C1x8, C2, C3, C4a-d, C5, C5m, and C5b,
C5bm: the second reading of configuration 5's layout; the masks run after both multiplies, so
that no operation directly follows the one that read the same inputs).  The operations touch about 3.5 GB of
distinct memory per step, so each one starts with a cold 256 MB Infinity Cache.  The timed
region runs the step K times with HIP events around the dominant operation only (`roofline`).
`per_op`: `avg_us` is the cold time per launch (the call on four sets of buffers in rotation,
one pair of events around the whole run - what a kernel trace shows too), `step_event_us` the
one-call event bracket in an untimed pass of the step (2-6 us more: event records and the
gaps they cause), `warm_us` the same buffers back to back, `host_us` the host time to plan and
enqueue one call, `plan_us` the planner alone through the binding.  `roofline_worst` is the
operation furthest below its own bar.  `next_ops` times what is built beyond the five
configurations, each call with cold caches.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--profile]

`--profile` runs the warm-up and the K steps and nothing else (no events, no repeat loops, no
other operations): the run to put under `rocprofv3 --kernel-trace`, so that every launch in the
trace is a launch of the step.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_all_cases.txt")


def _source_digest() -> str:
    """Fingerprint of the kernel and planner sources: measured HBM traffic is only reported
    while the code it was measured on is unchanged."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1810_08723_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hpp", ".hip", ".cpp", ".inl")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def _measured_traffic():
    """case -> HBM bytes per launch from the committed rocprofv3 counter summary, or {} when
    the sources changed since it was taken."""
    out = {}
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return out
    digest = None
    for ln in lines:
        if ln.startswith("source_digest:"):
            digest = ln.split(":", 1)[1].strip()
        if ln.startswith("traffic "):
            f = dict(kv.split("=") for kv in ln.split()[1:])
            out[f["case"]] = float(f["hbm_bytes"])
    return out if digest == _source_digest() else {}



def _device_cases(cases):
    """Upload every case's storages; returns a list of (case, callable, device tensors)."""
    import torch
    import paper_1810_08723_amd as ocn
    uploaded = {}

    def dev(view):
        key = id(view.storage)
        if key not in uploaded:
            uploaded[key] = torch.from_numpy(view.storage).to("cuda:0")
        return ocn.Tensor.on_storage(uploaded[key], view.dtype, view.sizes, view.strides, view.offset,
                                     view.byteswapped)

    runs = []
    for c in cases:
        ins = [dev(v) for v in c.inputs]
        out = dev(c.out)
        if c.kind == "binary":
            fn = (lambda ins=ins, out=out, c=c: ocn.binary(c.op, ins[0], ins[1], out))
        elif c.kind == "unary":
            fn = (lambda ins=ins, out=out, c=c: ocn.unary(c.op, ins[0], out))
        elif c.kind == "binary_reduce":
            need = ocn.binary_reduce_workspace_bytes(c.op, c.red_op, ins[0], ins[1], list(c.axes), out, c.mid_dtype)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")
            fn = (lambda ins=ins, out=out, c=c, ws=ws: ocn.binary_reduce(c.op, c.red_op, ins[0], ins[1], list(c.axes),
                                                                         out, c.mid_dtype, workspace=ws))
        else:
            need = ocn.reduce_workspace_bytes(c.op, ins[0], list(c.axes), out)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")
            fn = (lambda ins=ins, out=out, c=c, ws=ws: ocn.reduce(c.op, ins[0], list(c.axes), out, workspace=ws))
        runs.append((c, fn, out))
    return runs, uploaded


def _plan_kernel(c):
    import paper_1810_08723_amd as ocn

    def fake(view, base):
        return ocn.Tensor(base, view.dtype, view.sizes, view.strides, view.offset, 0, None, view.byteswapped)
    ins = [fake(v, 0x100000000 * (i + 1)) for i, v in enumerate(c.inputs)]
    out = fake(c.out, 0x700000000)
    if c.kind == "binary":
        return ocn.plan_binary(c.op, ins[0], ins[1], out)
    if c.kind == "unary":
        return ocn.plan_unary(c.op, ins[0], out)
    if c.kind == "binary_reduce":
        return ocn.plan_binary_reduce(c.op, c.red_op, ins[0], ins[1], list(c.axes), out, c.mid_dtype)
    return ocn.plan_reduce(c.op, ins[0], list(c.axes), out)


BAR = {"C2": 0.8, "C3": 0.8, "C4a": 0.8, "C4b": 0.8, "C4c": 0.8, "C4d": 0.8,
       "C1x8": 0.5, "C5": 0.5, "C5m": 0.5, "C5b": 0.5, "C5bm": 0.5}
"""Fraction of the HBM peak each case is held to: 0.8 for contiguous and broadcast elementwise
operations and reductions, 0.5 for permuted-stride cases.  C1 (1.2 MB) is bound by launch
latency and has no bandwidth bar."""

CPU_SAMPLE = ("C2", "C3", "C4a", "C4b", "C4c", "C4d")


def _oracle_call(c):
    from oracle import binding as O
    if c.kind == "binary":
        O.binary(c.op, c.inputs[0], c.inputs[1], c.out)
    elif c.kind == "unary":
        O.unary(c.op, c.inputs[0], c.out)
    else:
        O.reduce(c.op, c.inputs[0], list(c.axes), c.out)


def _cpu_baseline(cases):
    """Times the CPU oracle, as it stands, on the SAME full-size host inputs the GPU cases were
    uploaded from: the six contiguous / broadcast / reduction cases (C2, C3, C4a-d; the
    permuted cases are left out to bound the time).  One pass on a single thread, then three
    passes on all host threads, best pass kept.  GB/s of the same logical bytes."""
    import ctypes
    gomp = ctypes.CDLL("libgomp.so.1")
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    sample = [c for c in cases if c.name in CPU_SAMPLE]
    if not sample:
        return None
    nbytes = sum(c.logical_bytes for c in sample)

    def one_pass():
        per = {}
        for c in sample:
            t = time.perf_counter()
            _oracle_call(c)
            per[c.name] = time.perf_counter() - t
        return per

    gomp.omp_set_num_threads(1)
    single = one_pass()
    gomp.omp_set_num_threads(threads)
    multi = [one_pass() for _ in range(3)]
    best = {k: min(m[k] for m in multi) for k in single}
    return {"value": nbytes / sum(best.values()) / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "single_thread_value": nbytes / sum(single.values()) / 1e9,
            "per_case_gbs": {c.name: {"threads_1": c.logical_bytes / single[c.name] / 1e9,
                                      f"threads_{threads}": c.logical_bytes / best[c.name] / 1e9} for c in sample},
            "sample": f"the full-size inputs of {', '.join(c.name for c in sample)} ({nbytes / 1e6:.0f} MB logical per "
                      f"pass): 1 pass on one thread, best of 3 passes on {threads} threads (the oracle's OpenMP loop "
                      "runs over output elements, so the single-output C4d stays on one thread)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile", action="store_true",
                    help="warm-up and the step loop only (the run to trace with rocprofv3)")
    ap.add_argument("--only", default="", help="comma-separated case names (for profiling one kernel); "
                    "'copy' adds a plain 1 GiB float copy used to calibrate the HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this engine runs on one GPU; --gpus must be 1 (nothing here is distributed)",
              file=sys.stderr)
        return 2

    import torch
    import paper_1810_08723_amd as ocn  # noqa: F401  (fails loudly if libocn.so is missing)
    from workloads import configs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3

    cases = configs.all_cases_full()
    if args.only:
        want = args.only.split(",")
        if any(w.startswith("F") for w in want):
            cases = cases + configs.fused_cases()
        if any(w[0] in "LS" for w in want):
            cases = cases + configs.layout_cases()
        if any(w.startswith("E") for w in want):
            cases = cases + configs.elementary_cases()
        cases = [c for c in cases if c.name in want]
        if "copy" in want:
            from workloads.views import View
            n = 1 << 28
            src = View.from_numpy(np.ones(n, dtype=np.float32))
            cases.append(configs.Case("copy", "unary", "ident", [src], View.empty("float", (n,)),
                                      logical_bytes=8 * n, note="plain contiguous copy (counter calibration)"))
    runs, _keep = _device_cases(cases)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        for _, fn, _ in runs:
            fn()
    torch.cuda.synchronize()

    if args.profile:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            for _, fn, _ in runs:
                fn()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        step_bytes = sum(c.logical_bytes for c in cases)
        print(json.dumps({"metric": "effective GB/s (logical bytes moved) and % of MI355X HBM peak per op",
                          "value": step_bytes * args.steps / wall / 1e9, "unit": "GB/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
                          "profile_run": True, "launches_per_case": args.steps + args.warmup,
                          "cases": [{"case": c.name, "logical_bytes": c.logical_bytes,
                                     "kernel": _plan_kernel(c)["kernel"], "grid": int(_plan_kernel(c)["grid"]),
                                     "block": int(_plan_kernel(c)["block"]),
                                     "passes": int(_plan_kernel(c)["passes"])} for c in cases]}))
        return 0

    # Untimed pass with HIP events around every call (recorded on the stream the kernels are
    # launched on: torch's current stream is passed to the library): per-operation device time
    # in the step, and which operation dominates.  Event records cost a few microseconds each,
    # so the timed region below brackets only the dominant operation.
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in runs] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for s in range(args.steps):
        for i, (_, fn, _) in enumerate(runs):
            ev[s][i][0].record()
            fn()
            ev[s][i][1].record()
    torch.cuda.synchronize()
    op_ms = [sorted(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)) for i in range(len(runs))]
    dom_i = max(range(len(runs)), key=lambda i: sum(op_ms[i]))

    # Cold, steady-state time per launch of every operation: the same call on four distinct sets
    # of buffers used in rotation (well over 256 MB between two uses of a buffer, so nothing is
    # found in the Infinity Cache again), one pair of events around the whole run of launches.
    # This is what the kernel durations of a rocprofv3 trace of the step show as well; the
    # one-call brackets above read 2-6 us more (event records and the launch gaps they cause).
    NB = 4
    sets = [runs] + [_device_cases(cases)[0] for _ in range(NB - 1)]
    torch.cuda.synchronize()
    cold_us = []
    for i in range(len(runs)):
        fns = [sets[k][i][1] for k in range(NB)]
        # a run of about 20 ms, entered without a pause after three untimed rounds (a shorter
        # run that starts on an idle device reads up to 15 % more: clocks, first touches)
        rounds = max(6, int(20e3 / (NB * max(op_ms[i][len(op_ms[i]) // 2] * 1e3, 1.0))))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            for f in fns:
                f()
        e0.record()
        for _ in range(rounds):
            for f in fns:
                f()
        e1.record()
        torch.cuda.synchronize()
        cold_us.append(e0.elapsed_time(e1) * 1e3 / (rounds * NB))
    del sets
    torch.cuda.empty_cache()

    # timed region: exactly `steps` passes of the whole step, events around the dominant call only
    dev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        for i, (_, fn, _) in enumerate(runs):
            if i == dom_i:
                dev[s][0].record()
                fn()
                dev[s][1].record()
            else:
                fn()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom_ms = [a.elapsed_time(b) for a, b in dev]

    step_bytes = sum(c.logical_bytes for c in cases)
    per_op = []
    for i, (c, _, _) in enumerate(runs):
        ms = op_ms[i]
        avg = sum(ms) / len(ms)
        plan = _plan_kernel(c)
        per_op.append({"case": c.name, "op": c.op, "kernel": plan["kernel"], "passes": plan["passes"],
                       "logical_bytes": c.logical_bytes, "avg_us": cold_us[i],
                       "step_event_us": avg * 1e3, "step_event_min_us": ms[0] * 1e3,
                       "gbs": c.logical_bytes / (cold_us[i] * 1e-6) / 1e9,
                       "frac_of_peak": c.logical_bytes / (cold_us[i] * 1e-6) / 1e9 / HBM_PEAK_GBS})
    # outside the timed region: steady-state (cache-warm) device time, and host-side cost
    for i, (c, fn, _) in enumerate(runs):
        reps = 12
        wev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in wev:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        w = sorted(a.elapsed_time(b) for a, b in wev[2:])
        per_op[i]["warm_us"] = w[len(w) // 2] * 1e3
        t1 = time.perf_counter()
        for _ in range(50):
            fn()
        per_op[i]["host_us"] = (time.perf_counter() - t1) / 50 * 1e6
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(50):
            _plan_kernel(c)
        per_op[i]["plan_us"] = (time.perf_counter() - t1) / 50 * 1e6
    # the fused elementwise+reduce cases, outside the timed step: device time of the one fused
    # call and of the same result computed as two calls through a temporary tensor
    next_ops = []
    if not args.only:
        del runs, _keep
        torch.cuda.empty_cache()
        fcases = configs.fused_cases() + configs.elementary_cases() + configs.layout_cases()
        fruns, _fkeep = _device_cases(fcases)

        # every timed call starts with cold caches: 1 GiB of other memory is read in between
        # (by torch, outside the event bracket), which pushes the operands out of the
        # 256 MB Infinity Cache without leaving dirty lines behind
        filler = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")

        def timed(f, reps=12):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in evs:
                filler.sum()
                a.record(); f(); b.record()
            torch.cuda.synchronize()
            t = sorted(a.elapsed_time(b) for a, b in evs[2:])
            return t[len(t) // 2] * 1e3

        for (c, fn, out) in fruns:
            if c.kind != "binary_reduce":
                us = timed(fn)
                plan = _plan_kernel(c)
                next_ops.append({"case": c.name, "op": c.op, "note": c.note, "kernel": plan["kernel"], "fused": False,
                                 "passes": plan["passes"], "logical_bytes": c.logical_bytes, "us": us,
                                 "gbs": c.logical_bytes / (us * 1e-6) / 1e9,
                                 "frac_of_peak": c.logical_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                 "two_calls_us": None})
                continue
            ins = [ocn.Tensor.on_storage(_fkeep[id(v.storage)], v.dtype, v.sizes, v.strides, v.offset) for v in c.inputs]
            shape = tuple(c.inputs[0].sizes)
            mid_t = torch.empty(int(np.prod(shape)) * ocn.dtype_size(c.mid_dtype), dtype=torch.uint8, device="cuda:0")
            st = []
            acc = ocn.dtype_size(c.mid_dtype)
            for n in reversed(shape):
                st.insert(0, acc)
                acc *= n
            mid = ocn.Tensor.on_storage(mid_t, c.mid_dtype, shape, tuple(st), 0)
            need = ocn.reduce_workspace_bytes(c.red_op, mid, list(c.axes), out)
            ws2 = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")

            def two_calls(c=c, ins=ins, mid=mid, out=out, ws2=ws2):
                ocn.binary(c.op, ins[0], ins[1], mid)
                ocn.reduce(c.red_op, mid, list(c.axes), out, workspace=ws2)

            us = timed(fn)
            us2 = timed(two_calls)
            plan = _plan_kernel(c)
            next_ops.append({"case": c.name, "op": f"{c.red_op}({c.op})", "kernel": plan["kernel"], "fused": plan["fused"],
                             "passes": plan["passes"], "logical_bytes": c.logical_bytes, "us": us,
                             "gbs": c.logical_bytes / (us * 1e-6) / 1e9,
                             "frac_of_peak": c.logical_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                             "two_calls_us": us2})
    # boolean-mask selection a[mask] over 2^26 fp32 values with half of them selected: the mask
    # is compacted to offsets (three launches), then the elements are gathered
    if not args.only:
        n = 1 << 26
        rng = np.random.default_rng(configs.BASE_SEED + 70)
        mask_h = rng.random(n) < 0.5
        a_d = torch.from_numpy(rng.standard_normal(n, dtype=np.float32)).to("cuda:0")
        m_d = torch.from_numpy(mask_h.view(np.uint8)).to("cuda:0")
        count_h = int(mask_h.sum())
        offs_d = torch.empty(count_h, dtype=torch.int64, device="cuda:0")
        out_d = torch.empty(count_h, dtype=torch.float32, device="cuda:0")
        cnt_d = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        tm = ocn.Tensor(m_d.data_ptr(), "bool", (n,), (1,), 0, 0, m_d)
        ta = ocn.Tensor(a_d.data_ptr(), "float", (), (), 0, 0, a_d)
        to = ocn.Tensor(out_d.data_ptr(), "float", (count_h,), (4,), 0, 0, out_d)
        ws = torch.empty(8 * (n // 4096 + 2), dtype=torch.uint8, device="cuda:0")
        f_bind = lambda: ocn.mask_offsets(tm, [4], offs_d, cnt_d, workspace=ws)
        f_gather = lambda: ocn.gather(ta, offs_d, 0, 4 * (n - 1), to)
        us_b, us_g = timed(f_bind), timed(f_gather)
        assert int(cnt_d.cpu()[0]) == count_h
        for name, us, lb, note in (("G1", us_b, n + 8 * count_h, "mask -> offsets (count, scan, write)"),
                                   ("G2", us_g, 8 * count_h + 4 * n + 4 * count_h,
                                    "gather by offsets (every line of the source is touched)")):
            next_ops.append({"case": name, "op": note, "kernel": "index", "fused": False, "passes": 3 if name == "G1" else 1,
                             "logical_bytes": lb, "us": us, "gbs": lb / (us * 1e-6) / 1e9,
                             "frac_of_peak": lb / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "two_calls_us": None})
    device_ms = sum(p["avg_us"] for p in per_op) / 1e3
    dom = dict(per_op[dom_i])
    dom["avg_us"] = sum(dom_ms) / len(dom_ms) * 1e3          # one-call brackets inside the timed region
    dom["gbs"] = dom["logical_bytes"] / (dom["avg_us"] * 1e-6) / 1e9
    traffic = _measured_traffic()
    for p in per_op:
        p["hbm_traffic_bytes"] = traffic.get(p["case"])

    barred = [p for p in per_op if p["case"] in BAR]
    for p in barred:
        p["target_frac"] = BAR[p["case"]]
    worst = min(barred, key=lambda p: p["frac_of_peak"] / p["target_frac"]) if barred else None

    result = {
        "metric": "effective GB/s (logical bytes moved) and % of MI355X HBM peak per op",
        "value": step_bytes * args.steps / wall / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32/f64/i32/i8/f16/c64 (per case)", "data": "synthetic",
        "config": {"workload": ("all five configurations in one step: C1, C1x8, C2, C3, C4a-d, C5, C5b, C5m, C5bm"
                                if not args.only else "subset for profiling: " + args.only),
                   "logical_bytes_per_step": step_bytes, "device_ms_per_step": device_ms},
        "roofline": {"bound": "hbm", "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": dom["gbs"] / HBM_PEAK_GBS, "traffic": traffic.get(dom["case"]),
                     "kernel": f"{dom['kernel']} ({dom['case']})",
                     "bytes_per_launch": dom["logical_bytes"], "avg_us": dom["avg_us"]},
        "per_op": per_op,
        "next_ops": next_ops,
    }
    if worst is not None:
        # the case furthest below its own bar (its in-step event time, cold caches)
        result["roofline_worst"] = {"bound": "hbm", "achieved": worst["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": worst["frac_of_peak"], "target_frac": worst["target_frac"],
                                    "traffic": traffic.get(worst["case"]),
                                    "kernel": f"{worst['kernel']} ({worst['case']})",
                                    "bytes_per_launch": worst["logical_bytes"], "avg_us": worst["avg_us"]}
    if not args.no_cpu_baseline:
        base = _cpu_baseline(cases)
        if base is not None:
            result["cpu_baseline"] = base
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
