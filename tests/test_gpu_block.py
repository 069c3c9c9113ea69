"""GPU parity on one processor's row block with halo rows fetched from a host-resident table
(the shape of the largest workload at 1/32 of its size, same generator, same Epoch call sequence as
bench.py): halo index list and remapped CSR/CSC bit for bit, gathered rows bit for bit, sampled rows of
the forward and backward results and every element of the weight gradients within 1e-5 * sum|terms|.
Run twice: with the halo fetch overlapped with the owned-column products (two-step sparse product), and
with the fetch before each layer (one-step product).
"""
import numpy as np
import pytest

import oracle
from util import TOL_F32, check_bound, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=[(True, "push"), (False, "push"), (True, "pull"), (False, "pull")],
                ids=["overlapped", "sequential", "pull-overlapped", "pull-sequential"])
def blk(request):
    import torch
    import bench
    import paper_2212_05009_amd as gcn
    from workloads import configs, table as wtable
    dev = torch.device("cuda:0")
    say("generating a row block: 2^17 owned rows of a 2^20-vertex graph")
    w = configs.row_block(n_global=1 << 20, n_rows=1 << 17, n_halo=6 << 15)
    n, lo, hi = w["n"], w["row_lo"], w["row_hi"]
    og = oracle.graph_build(w["src"], w["dst"], n, lo, hi, deg_global=w["deg_global"])
    say(f"gpu block build rows={og.nr} halo={og.nh} nnz={og.nnz}")
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n, lo, hi,
                          deg_global=torch.from_numpy(w["deg_global"]).to(dev))
    tab = torch.empty((n, w["dims"][0]), dtype=torch.float32, pin_memory=True)
    wtable.fill_table_torch(tab, w["table_seed"], dev)
    Ws = [torch.from_numpy(m).to(dev) for m in w["W"]]
    ep = bench.Epoch(gcn, torch, A, tab[lo:hi].to(dev), Ws, torch.from_numpy(w["y"]).to(dev), False, table=tab,
                     overlap=request.param[0], backward=request.param[1])
    say(f"block epoch with halo gathers from the pinned host table, overlap={request.param}")
    ep.run()
    ep.run()
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    order = np.argsort(-og.deg.astype(np.int64), kind="stable")
    rows = np.unique(np.concatenate([order[:30], rng.integers(0, og.nr, 1200), [0, og.nr - 1]])).astype(np.int64)
    return {"w": w, "og": og, "A": A, "ep": ep, "rows": rows, "tab": tab, "wtable": wtable, "pull": request.param[1] == "pull"}


def test_block_arrays_and_halo_list_bit_exact(blk):
    og, A = blk["og"], blk["A"]
    assert (A.nr, A.nh, A.nnz) == (og.nr, og.nh, og.nnz) and og.nh > 100000
    arr = A.arrays()
    for name in ["rowptr", "col", "deg", "halo_gid", "colptr", "rowidx"]:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name


def test_block_gathered_rows_bit_exact(blk):
    w, og, ep = blk["w"], blk["og"], blk["ep"]
    d = w["dims"][0]
    assert np.array_equal(blk["tab"][:4096].numpy(), blk["wtable"].table_rows(np.arange(4096), d, w["table_seed"]))
    want = blk["wtable"].table_rows(og.halo_gid, d, w["table_seed"])          # recomputed on the CPU, row by row
    for k in range(2):
        assert np.array_equal(ep.H[k][og.nr:].cpu().numpy(), want), f"halo rows of layer input {k}"
    own = blk["wtable"].table_rows(np.arange(w["row_lo"], w["row_hi"]), d, w["table_seed"])
    assert np.array_equal(ep.H[0][: og.nr].cpu().numpy(), own)


def test_block_forward_and_backward(blk):
    w, og, ep, rows = blk["w"], blk["og"], blk["ep"], blk["rows"]
    W1, W2 = (m.astype(np.float64) for m in w["W"])
    H0 = ep.H[0].cpu().numpy()
    AX, BAX = oracle.spmm(og.rowptr, og.col, og.val, H0, rows=rows)
    Z1, B1 = AX @ W1, BAX @ np.abs(W1)
    check_bound(ep.H[1][rows].cpu().numpy(), np.maximum(Z1, 0), B1, TOL_F32, "H1 rows")
    H1 = ep.H[1].cpu().numpy()                      # owned rows from layer 1, halo rows from the table
    AH, BAH = oracle.spmm(og.rowptr, og.col, og.val, H1)
    check_bound(ep.Zlast.cpu().numpy()[rows], AH[rows] @ W2, BAH[rows] @ np.abs(W2), TOL_F32, "Z2 rows")
    Z2 = ep.Zlast.cpu().numpy()
    loss, labs, G = oracle.softmax_xent(Z2, w["y"], 1.0 / og.nr)
    assert abs(float(ep.loss.item()) - loss) <= TOL_F32 * max(labs, np.abs(Z2).max() * 3)
    if blk["pull"]:
        return backward_pull_checks(blk, G, H0, H1)
    G2 = ep.G[1].cpu().numpy()
    onehot = np.zeros_like(G); onehot[np.arange(og.nr), w["y"]] = 1.0 / og.nr
    check_bound(G2, G, G + 2 * onehot, TOL_F32, "G2")
    G2d = G2.astype(np.float64)
    check_bound(ep.dW[1].cpu().numpy(), AH.T @ G2d, BAH.T @ np.abs(G2d), TOL_F32, "dW2")
    # dH over all local columns: owned rows masked by [H1 > 0], halo rows (contributions owed elsewhere) not
    cols = np.unique(np.concatenate([rows, og.nr + np.arange(0, og.nh, 97)])).astype(np.int64)
    T, BT = oracle.spmm(og.colptr, og.rowidx, og.val_t, G2, rows=cols)
    S, BS = T @ W2.T, BT @ np.abs(W2.T)
    own = cols < og.nr
    S[own] = np.where(H1[cols[own]] > 0, S[own], 0.0)
    check_bound(ep.D[0][cols].cpu().numpy(), S, BS, TOL_F32, "dH rows (owned and halo)")
    G1 = ep.G[0].cpu().numpy().astype(np.float64)
    AXf, BAXf = oracle.spmm(og.rowptr, og.col, og.val, H0)
    check_bound(ep.dW[0].cpu().numpy(), AXf.T @ G1, BAXf.T @ np.abs(G1), TOL_F32, "dW1")


def backward_pull_checks(blk, G, H0, H1):
    """Algorithm 2 on the block: halo rows of G^k from the table, T = A^ [G; G_halo], dH (owned rows, complete), dW."""
    w, og, ep = blk["w"], blk["og"], blk["ep"]
    W1, W2 = w["W"]
    C = w["dims"][2]
    want_halo = blk["wtable"].table_rows(og.halo_gid, w["dims"][0], w["table_seed"])
    D2 = ep.D[1].cpu().numpy()
    onehot = np.zeros_like(G); onehot[np.arange(og.nr), w["y"]] = 1.0 / og.nr
    check_bound(D2[: og.nr], G, G + 2 * onehot, TOL_F32, "G2 (owned rows)")
    assert np.array_equal(D2[og.nr:], want_halo[:, :C]), "halo rows of G2"
    b2 = oracle.layer_bwd_pull(og, H1[: og.nr], W2, D2, Zprev=H1[: og.nr])
    check_bound(ep.T[1].cpu().numpy(), b2["T"], b2["BT"], TOL_F32, "T2")
    check_bound(ep.dW[1].cpu().numpy(), b2["dW"], b2["BdW"], TOL_F32, "dW2 (pull)")
    D1 = ep.D[0].cpu().numpy()
    check_bound(D1[: og.nr], b2["dH"], b2["BdH"], TOL_F32, "G1 (owned rows)")
    assert np.array_equal(D1[og.nr:], want_halo), "halo rows of G1"
    b1 = oracle.layer_bwd_pull(og, H0[: og.nr], W1, D1)
    check_bound(ep.T[0].cpu().numpy(), b1["T"], b1["BT"], TOL_F32, "T1")
    check_bound(ep.dW[0].cpu().numpy(), b1["dW"], b1["BdW"], TOL_F32, "dW1 (pull)")
