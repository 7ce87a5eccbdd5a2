"""The single-launch paths recorded into a HIP graph and replayed.

The fused path of expm() (matrices that fit a compute unit) and expm_lowrank() enqueue kernels only: no host
read-back, no memset, no allocation once the workspace is reserved.  A caller with a launch-bound loop (many small
batches per step, as in a flow model) can therefore record them into a graph.  Every replay is checked bit for bit
against an eager call on the same input, with eager work and synchronisations between the replays.
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
