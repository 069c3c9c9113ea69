"""GPU parity: gcn_csr_induced (Sec. 4.3.3: a mini-batch is an induced subgraph treated as a graph of its own)
and mini-batch training steps on a directed graph against the oracle.

Structure arrays and values must be bit-identical to the oracle's build of the relabelled edge list
(integer work; values are one fp32 product of two correctly rounded factors on both sides).  The
sampler is the tests' own (uniform distinct vertices, seeded): the paper does not fix one.
"""
import numpy as np
import pytest

import oracle
from util import hub_graph, say

pytestmark = pytest.mark.gpu
NAMES = ["rowptr", "col", "deg", "colptr", "rowidx"]


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def dev_i32(a, dev):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)


def check_induced(gcn, dev, A, src, dst, n, V):
    og = oracle.graph_build(*oracle.induced_edges(src, dst, n, V), len(V))
    say(f"csr_induced n={n} n_sub={len(V)} nnz_sub={og.nnz}")
    B = gcn.gcn_csr_induced(A, dev_i32(V, dev))
    assert (B.nr, B.nh, B.nnz) == (og.nr, 0, og.nnz)
    arr = B.arrays()
    for name in NAMES:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name
    return og, B


@pytest.mark.parametrize("n,m,k,directed,seed", [
    (64, 300, 1, True, 1), (500, 4000, 37, True, 2), (5000, 60000, 1000, False, 3), (30000, 400000, 30000, True, 4),
    (30000, 400000, 4096, False, 5), (100000, 2000000, 25000, True, 6)])
def test_induced_matches_oracle(gcn, dev, n, m, k, directed, seed):
    rng = np.random.default_rng(seed)
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    src, dst = (u, v) if directed else (np.r_[u, v], np.r_[v, u])
    A = gcn.gcn_csr_build(dev_i32(src, dev), dev_i32(dst, dev), n)
    V = rng.permutation(n)[:k]
    check_induced(gcn, dev, A, src, dst, n, V)
    check_induced(gcn, dev, A, src, dst, n, np.sort(V))


def test_induced_with_hub_rows(gcn, dev):
    src, dst = hub_graph(9000, 3, 6.0, seed=21)
    A = gcn.gcn_csr_build(dev_i32(src, dev), dev_i32(dst, dev), 9000)
    rng = np.random.default_rng(2)
    V = np.unique(np.r_[[0, 1, 2], rng.permutation(9000)[:6000]])
    og, _ = check_induced(gcn, dev, A, src, dst, 9000, V)
    assert og.deg.max() > 2048


def test_induced_argument_errors(gcn, dev):
    import torch
    rng = np.random.default_rng(3)
    n = 200
    src, dst = rng.integers(0, n, 900), rng.integers(0, n, 900)
    A = gcn.gcn_csr_build(dev_i32(src, dev), dev_i32(dst, dev), n)
    for bad in ([3, 7, 3], [0, 200], [-1, 5], []):
        with pytest.raises(gcn.GcnError):
            gcn.gcn_csr_induced(A, dev_i32(np.array(bad, np.int32), dev))
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_induced(A, dev_i32(np.arange(n + 1) % n, dev))
    blk = gcn.gcn_csr_build(dev_i32(src, dev), dev_i32(dst, dev), n, 20, 90, deg_global=A.arrays()["deg"])
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_induced(blk, dev_i32([1, 2], dev))
    torch.cuda.synchronize()


def test_minibatch_training_on_a_directed_graph(gcn, dev):
    """Three mini-batches of a directed graph (A^^T != A^): subgraph build, feature and label rows fetched
    through the vertex list, forward, loss, backward through the column-major copy, update - losses and final
    weights against the oracle's loop run on its own subgraphs."""
    import torch
    rng = np.random.default_rng(11)
    n, m, dims, lr = 6000, 50000, [24, 16, 5], 0.5
    src, dst = rng.integers(0, n, m), rng.integers(0, n, m)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[2], n).astype(np.int32)
    W0 = [(rng.standard_normal((dims[k], dims[k + 1])) / np.sqrt(dims[k])).astype(np.float32) for k in range(2)]
    batches = [rng.permutation(n)[:1500] for _ in range(3)]

    Wo, want = [w.copy() for w in W0], []
    for V in batches:
        og = oracle.graph_build(*oracle.induced_edges(src, dst, n, V), len(V))
        assert not np.array_equal(og.col, og.rowidx)              # the batch graph really is asymmetric
        losses, Wo = oracle.train(og, X[V], Wo, y[V], lr, 1)
        want.append(losses[0])

    A = gcn.gcn_csr_build(dev_i32(src, dev), dev_i32(dst, dev), n)
    Xd = torch.from_numpy(X).to(dev)
    yd = torch.from_numpy(y.view(np.float32).reshape(n, 1).copy()).to(dev)       # labels ride the row gather as 4-byte rows
    Ws = [torch.from_numpy(w.copy()).to(dev) for w in W0]
    dWs = [torch.empty_like(w) for w in Ws]
    loss = torch.zeros(1, device=dev)
    got = []
    for V in batches:
        k = len(V)
        Vd = dev_i32(V, dev)
        say(f"mini-batch of {k} vertices")
        B = gcn.gcn_csr_induced(A, Vd)
        Xb = torch.empty(k, dims[0], device=dev); yb = torch.empty(k, 1, device=dev)
        gcn.gcn_halo_gather(Xd, Vd, Xb)
        gcn.gcn_halo_gather(yd, Vd, yb)
        H1 = torch.empty(k, dims[1], device=dev); Z2 = torch.empty(k, dims[2], device=dev)
        G2 = torch.empty_like(Z2); G1 = torch.empty_like(H1)
        gcn.gcn_layer_fwd(B, Xb, Ws[0], H1, act=gcn.ACT_RELU)
        gcn.gcn_layer_fwd(B, H1, Ws[1], Z2, act=gcn.ACT_NONE)
        gcn.gcn_softmax_xent(Z2, yb.view(torch.int32).reshape(k), 1.0 / k, loss, G2)
        got.append(float(loss.item()))
        gcn.gcn_layer_bwd(B, H1, Ws[1], G2, dWs[1], dH=G1, Zprev=H1)
        gcn.gcn_layer_bwd(B, Xb, Ws[0], G1, dWs[0])
        for W, dW in zip(Ws, dWs):
            gcn.gcn_sgd_update(W, dW, lr)
        torch.cuda.synchronize()
        B.free()
    for e, (a, b) in enumerate(zip(got, want)):
        assert abs(a - b) <= 1e-5 * (1 + e) * abs(b), (e, a, b)
    for W, Wref in zip(Ws, Wo):
        assert np.max(np.abs(W.cpu().numpy() - Wref)) <= 1e-4
