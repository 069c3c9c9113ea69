"""GPU parity at the benchmark's full size (R-MAT 2^18, average degree 50, 128 -> 128 -> 16), in the launch
configuration bench.py times: the same Epoch call sequence, then

  * the whole CSR / CSC / degree arrays, bit for bit;
  * sampled output rows (longest rows, random rows, first and last) of every row-wise result, each
    recomputed by the oracle from the GPU's own inputs of that call;
  * every element of the weight gradients, whose sums run over all rows: the oracle's sparse product
    followed by an fp64 matrix product (a library routine used as one step of the definition).

Tolerance as everywhere: |gpu - oracle| <= 1e-5 * (the same sum with absolute values).
"""
import numpy as np
import pytest

import oracle
from util import TOL_F32, check_bound, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def full():
    import torch
    import bench
    import paper_2212_05009_amd as gcn
    from workloads import configs
    dev = torch.device("cuda:0")
    say("generating the full-size workload")
    w = configs.get("c2_rmat18")
    n = w["n"]
    say(f"oracle graph build n={n} raw edges={w['src'].size}")
    og = oracle.graph_build(w["src"], w["dst"], n)
    say("gpu graph build")
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n)
    X = torch.from_numpy(w["X"]).to(dev)
    Ws = [torch.from_numpy(m).to(dev) for m in w["W"]]
    y = torch.from_numpy(w["y"]).to(dev)
    ep = bench.Epoch(gcn, torch, A, X, Ws, y, False)
    say("epoch (forward, loss, backward) as bench.py runs it")
    ep.run()
    ep.run()
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    order = np.argsort(-og.deg.astype(np.int64), kind="stable")
    rows = np.unique(np.concatenate([order[:40], order[-5:], rng.integers(0, n, 1500), [0, n - 1]])).astype(np.int64)
    return {"w": w, "og": og, "A": A, "ep": ep, "rows": rows, "gcn": gcn, "torch": torch}


def test_fullsize_graph_arrays_bit_exact(full):
    og, A = full["og"], full["A"]
    assert (A.nr, A.nh, A.nnz) == (og.nr, 0, og.nnz)
    arr = A.arrays()
    for name in ["rowptr", "col", "deg", "colptr", "rowidx"]:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name
    assert og.deg.max() > 2048          # the chunked long-row path is exercised at this size


def test_fullsize_forward_rows(full):
    w, og, ep, rows = full["w"], full["og"], full["ep"], full["rows"]
    W1, W2 = (m.astype(np.float64) for m in w["W"])
    # layer 1: Z1 = (A^ X) W1, H1 = relu(Z1)
    AX, BAX = oracle.spmm(og.rowptr, og.col, og.val, w["X"], rows=rows)
    Z1, B1 = AX @ W1, BAX @ np.abs(W1)
    check_bound(ep.H[1][rows].cpu().numpy(), np.maximum(Z1, 0), B1, TOL_F32, "H1 rows")
    assert float(ep.H[1].min()) == 0.0           # ReLU applied
    # layer 2 from the GPU's H1: Z2 = A^ (H1 W2) in the library, the same sum as (A^ H1) W2
    H1 = ep.H[1].cpu().numpy()
    AH, BAH = oracle.spmm(og.rowptr, og.col, og.val, H1, rows=rows)
    check_bound(ep.Zlast[rows].cpu().numpy(), AH @ W2, BAH @ np.abs(W2), TOL_F32, "Z2 rows")
    # the saved A^ X of layer 1
    check_bound(ep.AH[0][rows].cpu().numpy(), AX, BAX, TOL_F32, "saved A^X rows")


def test_fullsize_loss_and_output_gradient(full):
    w, ep = full["w"], full["ep"]
    n = w["n"]
    Z2 = ep.Zlast.cpu().numpy()
    loss, labs, G = oracle.softmax_xent(Z2, w["y"], 1.0 / n)
    assert abs(float(ep.loss.item()) - loss) <= TOL_F32 * max(labs, np.abs(Z2).max() * 3)
    onehot = np.zeros_like(G); onehot[np.arange(n), w["y"]] = 1.0 / n
    check_bound(ep.G[1].cpu().numpy(), G, G + 2 * onehot, TOL_F32, "G2")


def test_fullsize_backward(full):
    w, og, ep, rows = full["w"], full["og"], full["ep"], full["rows"]
    W2 = w["W"][1].astype(np.float64)
    H1 = ep.H[1].cpu().numpy()
    Z1 = H1          # the epoch takes the ReLU mask from H1 = max(Z1, 0): positive exactly where Z1 is
    G2 = ep.G[1].cpu().numpy()
    # dW2 = (A^ H1)^T G2, every element
    AH, BAH = oracle.spmm(og.rowptr, og.col, og.val, H1)
    G2d = G2.astype(np.float64)
    check_bound(ep.dW[1].cpu().numpy(), AH.T @ G2d, BAH.T @ np.abs(G2d), TOL_F32, "dW2")
    # G1 rows = (A^T G2 W2^T) * [Z1 > 0]
    T, BT = oracle.spmm(og.colptr, og.rowidx, og.val_t, G2, rows=rows)
    S, BS = T @ W2.T, BT @ np.abs(W2.T)
    S[~(Z1[rows] > 0)] = 0.0
    check_bound(ep.G[0][rows].cpu().numpy(), S, BS, TOL_F32, "G1 rows")
    # dW1 = (A^ X)^T G1 with the GPU's G1 and the oracle's own A^ X, every element
    G1 = ep.G[0].cpu().numpy().astype(np.float64)
    AX, BAX = oracle.spmm(og.rowptr, og.col, og.val, w["X"])
    check_bound(ep.dW[0].cpu().numpy(), AX.T @ G1, BAX.T @ np.abs(G1), TOL_F32, "dW1")
