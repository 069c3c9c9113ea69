"""A whole epoch of library calls captured into a HIP graph (torch.cuda.CUDAGraph) and replayed.

The calls of an epoch only enqueue kernels on the caller's stream (no allocation, copy or memset node once the handle's
workspace has its size), so a latency-bound epoch can be replayed as one graph launch.  Every replay must give, bit for
bit, what the same calls give eagerly; eager epochs and synchronisations sit between the replays.
"""
import numpy as np
import pytest

from util import say, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


def _snapshot(ep):
    return [to_np(ep.loss).copy(), to_np(ep.Zlast).copy()] + [to_np(dW).copy() for dW in ep.dW] + \
           [to_np(d).copy() for d in ep.D]


def test_epoch_replayed_from_a_graph(gcn, c1):
    import torch
    import bench
    dev = torch.device("cuda:0")
    w = c1
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), w["n"])
    Ws = [torch.from_numpy(m.copy()).to(dev) for m in w["W"]]
    ep = bench.Epoch(gcn, torch, A, torch.from_numpy(w["X"]).to(dev), Ws, torch.from_numpy(w["y"]).to(dev), False)
    say("eager epochs (the workspace takes its size)")
    for _ in range(2):
        ep.run()
    torch.cuda.synchronize()
    want = _snapshot(ep)
    graph = torch.cuda.CUDAGraph()
    say("capture")
    with torch.cuda.graph(graph):
        ep.run()
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work of the program's own between the replays: other weights, so that every buffer is overwritten
        for W in Ws:
            W.mul_(-0.5)
        ep.run()
        torch.cuda.synchronize()
        assert not np.array_equal(_snapshot(ep)[1], want[1])
        for W in Ws:
            W.mul_(-2.0)
        torch.cuda.synchronize()
        say(f"replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        got = _snapshot(ep)
        for a, b in zip(got, want):
            assert np.array_equal(a, b), f"replay {rep} differs from the eager epoch"
    A.free()


def test_layer_calls_with_the_second_stream_replayed_from_a_graph(gcn, c1):
    """The layer calls with dense products beside sparse ones (forced on for this small graph): the library's second
    stream joins the capture through the events that tie it to the caller's stream, and the replays equal the eager
    calls bit for bit."""
    import torch
    dev = torch.device("cuda:0")
    w = c1
    n, d = w["n"], 256
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n)
    torch.manual_seed(3)
    H = torch.randn(n, d, device=dev); W = torch.randn(d, d, device=dev) / 16.0; G = torch.randn(n, d, device=dev) / n
    Hout = torch.empty(n, d, device=dev); AH = torch.empty(n, d, device=dev)
    dW = torch.empty(d, d, device=dev); dH = torch.empty(n, d, device=dev)

    def calls():
        gcn.gcn_layer_fwd(A, H, W, Hout, act=gcn.ACT_RELU, AH_save=AH)
        gcn.gcn_layer_bwd(A, H, W, G, dW, dH=dH, Zprev=H, AH_saved=AH)

    for name, v in (("GCN_OVERLAP", 2), ("GCN_GEMM_REGW", 2), ("GCN_GEMM_TN_LDS", 2)):
        gcn.gcn_debug_set_tuning(name, v)
    try:
        say("eager calls (the second stream, its events and the workspace come into being)")
        for _ in range(2):
            calls()
        torch.cuda.synchronize()
        want = [to_np(t).copy() for t in (Hout, AH, dW, dH)]
        graph = torch.cuda.CUDAGraph()
        say("capture")
        with torch.cuda.graph(graph):
            calls()
        torch.cuda.synchronize()
        for rep in range(3):
            for t in (Hout, AH, dW, dH):
                t.zero_()
            torch.cuda.synchronize()
            say(f"replay {rep}")
            graph.replay()
            torch.cuda.synchronize()
            for a, b, what in zip((Hout, AH, dW, dH), want, ("Hout", "AH", "dW", "dH")):
                assert np.array_equal(to_np(a), b), f"replay {rep}: {what} differs from the eager calls"
    finally:
        for name in ("GCN_OVERLAP", "GCN_GEMM_REGW", "GCN_GEMM_TN_LDS"):
            gcn.gcn_debug_set_tuning(name, None)
        A.free()
