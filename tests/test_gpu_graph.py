"""Calls recorded into a HIP graph and replayed; calls on several streams.

Under stream capture expm() and expm_lowrank() enqueue kernels only: no host read-back, no memset, no other stream,
no allocation once the workspace is reserved.  A caller with a launch-bound loop (many small batches per step, as in
a flow model) can therefore record them into a graph.  Every replay is checked bit for bit against an eager call on
the same input, with eager work and synchronisations between the replays.
"""
import numpy as np
import pytest

from paper_2512_20777_amd import workloads


@pytest.fixture(scope="module")
def ex():
    import torch
    import paper_2512_20777_amd as ex
    assert torch.cuda.is_available(), "GPU tests need a device"
    ex.load_library()
    return ex


@pytest.mark.gpu
@pytest.mark.parametrize("n,batch,dtype", [(16, 1024, np.float32), (16, 1024, np.float64), (48, 96, np.float32),
                                           (96, 40, np.float64)])
def test_fused_expm_replayed_from_a_graph_equals_eager(ex, n, batch, dtype):
    import torch
    dt = ex.DTYPE_F64 if dtype == np.float64 else ex.DTYPE_F32
    first = workloads.random_stack(9100 + n, batch, n, dtype, 0.01, 10.0, "skew")
    static_in = torch.from_numpy(first).cuda()
    static_out = torch.empty_like(static_in)
    ex.expm_reserve(n, batch, dt)
    ex.expm(static_in, 0.0, out=static_out)       # first call outside the capture: attributes, workspace
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print("capture n=%d batch=%d %s" % (n, batch, np.dtype(dtype).name), flush=True)
    with torch.cuda.graph(graph, stream=side):
        ex.expm(static_in, 0.0, out=static_out)
    for rep in range(4):
        fresh = workloads.random_stack(9200 + 7 * rep + n, batch, n, dtype, 0.01, 10.0, "dense" if rep % 2 else "skew")
        static_in.copy_(torch.from_numpy(fresh).cuda())
        static_out.zero_()
        eager, st = ex.expm(static_in.clone(), 0.0)     # the program's own eager work between replays
        torch.cuda.synchronize()
        assert st == 0
        print("   replay %d" % rep, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(static_out, eager), (n, batch, rep)


@pytest.mark.gpu
def test_lowrank_replayed_from_a_graph_equals_eager(ex):
    import torch
    n, t, batch = 256, 32, 24
    a1, a2 = workloads.lowrank_stack(9300, batch, n, t, np.float32, 1e-3, 2.0)
    s1, s2 = torch.from_numpy(a1).cuda(), torch.from_numpy(a2).cuda()
    static_out = torch.empty((batch, n, n), dtype=s1.dtype, device="cuda")
    ex.expm_lowrank(s1, s2, 0.0, out=static_out)   # first call outside the capture: attributes, workspace
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print("capture low-rank n=%d t=%d batch=%d" % (n, t, batch), flush=True)
    with torch.cuda.graph(graph, stream=side):
        ex.expm_lowrank(s1, s2, 0.0, out=static_out)
    for rep in range(3):
        b1, b2 = workloads.lowrank_stack(9310 + rep, batch, n, t, np.float32, 1e-3, 2.0)
        s1.copy_(torch.from_numpy(b1).cuda())
        s2.copy_(torch.from_numpy(b2).cuda())
        static_out.zero_()
        eager, st = ex.expm_lowrank(s1.clone(), s2.clone(), 0.0)
        torch.cuda.synchronize()
        assert st == 0
        print("   replay %d" % rep, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(static_out, eager), rep


@pytest.mark.gpu
@pytest.mark.parametrize("n,batch,dtype,scheme", [(200, 5, np.float64, 0), (512, 3, np.float64, 0), (136, 6, np.float32, 0),
                                                  (200, 4, np.float64, 1), (512, 32, np.float64, 0), (1024, 8, np.float64, 0),
                                                  (1152, 8, np.float32, 1)])
def test_round_based_expm_replayed_from_a_graph_equals_eager(ex, n, batch, dtype, scheme):
    """Above the on-chip sizes the number of product rounds depends on the data.  Under capture the rounds are planned
    on the device (every possible round is recorded, workgroups of rounds a matrix does not need leave at once), so one
    graph serves inputs with different (m, s): each replay gets norms from another range."""
    import torch
    dt = ex.DTYPE_F64 if dtype == np.float64 else ex.DTYPE_F32
    static_in = torch.from_numpy(workloads.random_stack(9400 + n, batch, n, dtype, 0.5, 20.0)).cuda()
    static_out = torch.empty_like(static_in)
    ex.expm_reserve(n, batch, dt)
    ex.expm(static_in, 0.0, out=static_out, scheme=scheme)   # first call outside the capture: attributes, workspace
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print("capture n=%d batch=%d %s scheme %d" % (n, batch, np.dtype(dtype).name, scheme), flush=True)
    with torch.cuda.graph(graph, stream=side):
        ex.expm(static_in, 0.0, out=static_out, scheme=scheme)
    ranges = [(1e-9, 1e-3), (0.05, 2.0), (5.0, 300.0), (1e-3, 80.0)]
    for rep, (lo, hi) in enumerate(ranges):
        fresh = workloads.random_stack(9500 + 7 * rep + n, batch, n, dtype, lo, hi, "dense" if rep % 2 else "triu")
        static_in.copy_(torch.from_numpy(fresh).cuda())
        static_out.zero_()
        eager, st = ex.expm(static_in.clone(), 0.0, scheme=scheme)     # the program's own eager work between replays
        torch.cuda.synchronize()
        m_e, s_e, _ = ex.expm_select(static_in, 0.0, scheme=scheme)
        print("   replay %d: s up to %d" % (rep, int(s_e.max())), flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(static_out, eager), (n, batch, rep)


@pytest.mark.gpu
def test_capture_refuses_to_grow_the_workspace(ex):
    import torch
    ex.expm_shutdown()                    # drop the cached workspace: the capture below would have to allocate
    a = torch.from_numpy(workloads.random_stack(9600, 2, 160, np.float64, 0.5, 5.0)).cuda()
    out = torch.empty_like(a)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    lib = ex.load_library()
    with torch.cuda.graph(graph, stream=side):
        out.zero_()                       # so that the graph is not empty
        status = lib.expm(a.data_ptr(), 160, 2, ex.DTYPE_F64, 0.0, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert status == -6, status           # refused, nothing enqueued, the capture itself stays valid
    torch.cuda.synchronize()
    res, st = ex.expm(a, 0.0, out=out)    # and the library is usable afterwards
    torch.cuda.synchronize()
    assert st == 0 and bool(torch.isfinite(res).all())


@pytest.mark.gpu
def test_calls_on_two_streams_are_ordered_not_corrupted(ex):
    """All calls share one workspace per device: a call on another stream is ordered behind the previous call."""
    import torch
    a = torch.from_numpy(workloads.random_stack(9700, 6, 256, np.float64, 0.5, 40.0)).cuda()
    b = torch.from_numpy(workloads.random_stack(9701, 6, 256, np.float64, 0.5, 40.0)).cuda()
    ra, _ = ex.expm(a)
    ra = ra.clone()
    rb, _ = ex.expm(b)
    rb = rb.clone()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    oa, ob = torch.empty_like(a), torch.empty_like(b)
    for rep in range(3):
        oa.zero_(); ob.zero_()
        torch.cuda.synchronize()
        ex.expm(a, out=oa, stream=s1)
        ex.expm(b, out=ob, stream=s2)     # no synchronisation in between
        ex.expm(a, out=oa, stream=s1)
        torch.cuda.synchronize()
        assert torch.equal(oa, ra) and torch.equal(ob, rb), rep


@pytest.mark.gpu
def test_calls_from_two_host_threads_are_serialised(ex):
    """Entry points take a lock and order calls on different streams: two threads hammering the library with
    different inputs each get their own results."""
    import threading
    import torch
    a = torch.from_numpy(workloads.random_stack(9800, 5, 192, np.float64, 0.5, 40.0)).cuda()
    b = torch.from_numpy(workloads.random_stack(9801, 64, 48, np.float32, 0.5, 40.0)).cuda()
    ra = ex.expm(a)[0].clone()
    rb = ex.expm(b)[0].clone()
    torch.cuda.synchronize()
    errors = []

    def worker(x, ref, stream):
        try:
            out = torch.empty_like(x)
            for _ in range(6):
                out.zero_()
                ex.expm(x, out=out, stream=stream)
                stream.synchronize()
                if not torch.equal(out, ref):
                    errors.append("mismatch for shape %s" % (tuple(x.shape),))
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append(repr(e))

    t1 = threading.Thread(target=worker, args=(a, ra, torch.cuda.Stream()))
    t2 = threading.Thread(target=worker, args=(b, rb, torch.cuda.Stream()))
    t1.start(); t2.start(); t1.join(); t2.join()
    assert not errors, errors
