"""Stream behaviour of the library on the GPU: calls recorded into a HIP graph and replayed
with changing inputs, and independent chains of calls on two streams at once.  The library
allocates nothing and clears nothing behind the caller's back, so both must just work."""
import numpy as np
import pytest

import gpu_harness as H
from workloads.values import random_view, rng_for
from workloads.views import View

pytestmark = pytest.mark.gpu


def _oracle_chain(a, b, c, cast_out, red_out, full_out):
    from oracle import binding as O
    O.binary("add", a, b, c)                 # c = a + b^T      (tiled kernel)
    O.unary("ident", c, cast_out)            # int16 <- float   (rows kernel)
    O.reduce("sum", c, [0], red_out)         # column sums      (split, two launches)
    O.reduce("max", c, [0, 1], full_out)     # full reduction   (split, two launches)


def test_graph_capture_and_replay_with_new_inputs():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(14000)
    n0, n1 = 1536, 640
    a = random_view(rng, "float", (n0, n1), specials=False)
    b = random_view(rng, "float", (n1, n0), specials=False).permute(1, 0)
    c = View.empty("float", (n0, n1))
    cast_out = View.empty("int16", (n0, n1))
    red_out = View.empty("float", (n1,))
    full_out = View.empty("float", ())
    dv = H.DeviceViews()
    ta, tb, tc = dv.tensor(a), dv.tensor(b), dv.tensor(c)
    tcast, tred, tfull = dv.tensor(cast_out), dv.tensor(red_out), dv.tensor(full_out)
    ws1 = torch.empty(max(256, ocn.reduce_workspace_bytes("sum", tc, [0], tred)), dtype=torch.uint8, device="cuda:0")
    ws2 = torch.empty(max(256, ocn.reduce_workspace_bytes("max", tc, [0, 1], tfull)), dtype=torch.uint8, device="cuda:0")
    assert ocn.plan_reduce("sum", tc, [0], tred)["passes"] == 2
    assert ocn.plan_reduce("max", tc, [0, 1], tfull)["passes"] == 2

    def enqueue():
        ocn.binary("add", ta, tb, tc)
        ocn.cast_copy(tc, tcast)
        ocn.reduce("sum", tc, [0], tred, workspace=ws1)
        ocn.reduce("max", tc, [0, 1], tfull, workspace=ws2)

    enqueue()                                # eager once: warms up, and gives the reference
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()                            # recorded on the capture stream (torch's current stream)
    torch.cuda.synchronize()

    dev_a = dv._by_id[id(a.storage)][1]
    dev_b = dv._by_id[id(b.storage)][1]
    for replay in range(3):
        # new input values, uploaded by ordinary eager work between the replays
        a.storage[:] = random_view(rng, "float", (n0, n1), specials=False).storage
        b.storage[:] = random_view(rng, "float", (n1, n0), specials=False).storage
        dev_a.copy_(torch.from_numpy(a.storage))
        dev_b.copy_(torch.from_numpy(b.storage))
        for v in (c, cast_out, red_out, full_out):          # poison the outputs
            dv._by_id[id(v.storage)][1].fill_(0x5A)
        torch.cuda.synchronize()
        print("graph replay", replay, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got = [dv.download(v).copy() for v in (c, cast_out, red_out, full_out)]
        _oracle_chain(a, b, c, cast_out, red_out, full_out)
        assert H.storages_equal("float", got[0], c.storage)
        assert np.array_equal(got[1], cast_out.storage)
        x = c.to_numpy().astype(np.float64)
        bound = 1e-6 * np.abs(x).sum(axis=0)
        assert np.all(np.abs(got[2].view(np.float32).astype(np.float64) - red_out.storage.view(np.float32)) <= bound)
        assert np.array_equal(got[3], full_out.storage)


def test_two_streams_at_once():
    import torch
    import paper_1810_08723_amd as ocn
    rng = rng_for(14001)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for k in range(2):
        shape = (700 + 50 * k, 900)
        a = random_view(rng, "double", shape, specials=False)
        b = random_view(rng, "double", shape[::-1], specials=False).permute(1, 0)
        c = View.empty("double", shape)
        m = View.empty("bool", shape)
        s = View.empty("double", (shape[0],))
        dv = H.DeviceViews()
        t = [dv.tensor(v) for v in (a, b, c, m, s)]
        jobs.append((dv, (a, b, c, m, s), t))
    torch.cuda.synchronize()
    for rep in range(4):
        for k, (dv, views, t) in enumerate(jobs):
            st = streams[k].cuda_stream
            ocn.binary("mul", t[0], t[1], t[2], stream=st)
            ocn.binary("gt", t[2], t[0], t[3], stream=st)
            ocn.reduce("sum", t[2], [1], t[4], stream=st)
    torch.cuda.synchronize()
    from oracle import binding as O
    for dv, (a, b, c, m, s), t in jobs:
        got = [dv.download(v).copy() for v in (c, m, s)]
        O.binary("mul", a, b, c)
        O.binary("gt", c, a, m)
        O.reduce("sum", c, [1], s)
        assert H.storages_equal("double", got[0], c.storage)
        assert np.array_equal(got[1], m.storage)
        x = c.to_numpy()
        assert np.all(np.abs(got[2].view(np.float64) - s.storage.view(np.float64)) <= 1e-13 * np.abs(x).sum(axis=1) + 1e-300)


def test_split_reductions_on_side_streams_with_wrapper_allocated_workspaces():
    # Two chains of two-launch (split) reductions on two side streams, each call letting the
    # wrapper allocate its workspace.  The workspace of one call is dropped by the wrapper while
    # its second launch may still be pending; unless the block is recorded as in use on the side
    # stream, the allocator hands it to the other chain's next call and the partial results mix.
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    rng = rng_for(14003)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for k in range(2):
        n = (1 << 22) + 4099 * (k + 1)
        x = View.from_numpy(rng.integers(-128, 127, size=n, endpoint=True, dtype=np.int8))
        outs = [View.empty("int64", ()) for _ in range(6)]
        dv = H.DeviceViews()
        tx = dv.tensor(x)
        touts = [dv.tensor(o) for o in outs]
        plan = ocn.plan_reduce("sum", tx, [0], touts[0])
        assert plan["split"] > 1 and plan["passes"] == 2
        jobs.append((dv, x, outs, tx, touts))
    torch.cuda.synchronize()
    for rep in range(6):
        for k, (dv, x, outs, tx, touts) in enumerate(jobs):
            ocn.reduce("sum", tx, [0], touts[rep], stream=streams[k].cuda_stream)
    torch.cuda.synchronize()
    for dv, x, outs, tx, touts in jobs:
        want = View.empty("int64", ())
        O.reduce("sum", x, [0], want)
        for o in outs:
            assert np.array_equal(dv.download(o), want.storage)


def test_graph_of_fused_reduce_mask_compaction_gather_and_domain_check():
    # the later entry points under capture: every buffer (outputs, workspaces, the count) is
    # allocated before the capture, the calls only launch kernels.  Each replay is compared
    # with the oracle on the inputs of that replay; ordinary eager work runs in between.
    import torch
    import paper_1810_08723_amd as ocn
    from oracle import binding as O
    from oracle import indexing as OI
    rng = rng_for(14002)
    n0, n1 = 96, 200
    a = random_view(rng, "float", (n0, n1), specials=False)
    b = random_view(rng, "float", (n0, n1), specials=False)
    dots = View.empty("float", (n0,))            # row-wise inner products, one fused kernel
    total = View.empty("int64", ())              # count of a > b over everything: split, two launches
    mask = View.empty("bool", (n0, n1))
    dv = H.DeviceViews()
    ta, tb, tdots, ttotal, tmask = (dv.tensor(v) for v in (a, b, dots, total, mask))
    dev = "cuda:0"
    ws_d = torch.empty(max(256, ocn.binary_reduce_workspace_bytes("mul", "sum", ta, tb, [1], tdots, "float")), dtype=torch.uint8, device=dev)
    ws_t = torch.empty(max(256, ocn.binary_reduce_workspace_bytes("gt", "sum", ta, tb, [0, 1], ttotal, "bool")), dtype=torch.uint8, device=dev)
    offs = torch.full((n0 * n1,), -1, dtype=torch.int64, device=dev)
    count = torch.zeros(1, dtype=torch.int64, device=dev)
    ws_m = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    picked = torch.zeros(n0 * n1, dtype=torch.float32, device=dev)
    tpicked = ocn.Tensor.on_storage(picked.view(torch.uint8), "float", (n0 * n1,), (4,))
    inner = ocn.Tensor.on_storage(dv._by_id[id(a.storage)][1], "float", (), ())
    flag = torch.zeros(1, dtype=torch.bool, device=dev)
    ws_f = torch.empty(1 << 16, dtype=torch.uint8, device=dev)

    def enqueue():
        ocn.binary_reduce("mul", "sum", ta, tb, [1], tdots, "float", workspace=ws_d)
        ocn.binary_reduce("gt", "sum", ta, tb, [0, 1], ttotal, "bool", workspace=ws_t)
        ocn.binary("gt", ta, tb, tmask)
        ocn.mask_offsets(tmask, (n1 * 4, 4), offs, count, workspace=ws_m)
        ocn.gather(inner, offs, 0, (n0 * n1 - 1) * 4, tpicked)    # offsets past the count are -1: skipped
        ocn.domain_check("sqrt", ta, flag, workspace=ws_f)

    enqueue()                                    # eager once (also resolves the library's device constants)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    torch.cuda.synchronize()
    dev_a, dev_b = dv._by_id[id(a.storage)][1], dv._by_id[id(b.storage)][1]
    for replay in range(3):
        fresh = random_view(rng, "float", (n0, n1), specials=False)
        a.storage[:] = fresh.storage
        if replay == 1:                          # no negative value: the square root's domain check must say so
            a.storage[:] = np.abs(a.to_numpy()).view(np.uint8).reshape(-1)
        b.storage[:] = random_view(rng, "float", (n0, n1), specials=False).storage
        dev_a.copy_(torch.from_numpy(a.storage))
        dev_b.copy_(torch.from_numpy(b.storage))
        offs.fill_(-1)
        picked.fill_(-7.0)
        torch.cuda.synchronize()
        print("graph replay", replay, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        O.binary_reduce("mul", "sum", a, b, [1], dots, "float")
        x = (a.to_numpy().astype(np.float64) * b.to_numpy().astype(np.float64))
        got_dots = dv.download(dots).view(np.float32).astype(np.float64)
        assert np.all(np.abs(got_dots - dots.storage.view(np.float32)) <= 2e-6 * np.abs(x).sum(axis=1))
        O.binary_reduce("gt", "sum", a, b, [0, 1], total, "bool")
        assert np.array_equal(dv.download(total), total.storage)
        O.binary("gt", a, b, mask)
        want_offs = OI.mask_offsets(mask, (n1 * 4, 4))
        n = int(count.cpu()[0])
        assert n == len(want_offs) == int(total.storage.view(np.int64)[0])
        assert np.array_equal(offs.cpu().numpy()[:n], want_offs)
        got_picked = picked.cpu().numpy()
        assert np.array_equal(got_picked[:n], a.to_numpy().reshape(-1)[want_offs // 4]) and np.all(got_picked[n:] == -7.0)
        assert bool(flag.cpu()[0]) == bool((a.to_numpy() < 0).any()) == (replay != 1)
