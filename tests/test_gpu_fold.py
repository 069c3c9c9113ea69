"""GPU parity with launches folded into two grid dimensions.

A launch whose x extent reaches 2^32 threads is not refused by the runtime: it runs with the thread count taken
modulo 2^32.  The library therefore caps a grid's x dimension and puts the rest in y.  Real inputs only reach the
second dimension beyond some 10^9 rows or entries; gcn_debug_max_grid_x lowers the cap so that the same code runs
here on small inputs: every kernel whose grid grows with the problem (graph build, both sparse products with
their long-row chunks, gather, padded copies, weight update, subgraph extraction, partition statistics) is
compared with the oracle as in the other test files, at a cap of 61 blocks (odd, so that a row of the grid does not
hold whole groups of feature slices).
"""
import numpy as np
import pytest

import oracle
from util import TOL_F32, check_bound, hub_graph, say, to_dev, to_np

import test_gpu_build as tb
import test_gpu_induced as ti
import test_gpu_layer as tl
import test_gpu_partition as tp
import test_gpu_parts as tparts

pytestmark = pytest.mark.gpu
CAP = 61


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


@pytest.fixture(autouse=True)
def folded(gcn):
    gcn.gcn_debug_max_grid_x(CAP)
    yield
    gcn.gcn_debug_max_grid_x(0)


def test_cap_argument(gcn):
    for bad in (-1, (1 << 22) + 1):
        with pytest.raises(gcn.GcnError):
            gcn.gcn_debug_max_grid_x(bad)
    gcn.gcn_debug_max_grid_x(1 << 22)
    gcn.gcn_debug_max_grid_x(CAP)


def test_build_folded(gcn, dev):
    src, dst = hub_graph(9000, 3, 6.0, seed=3)
    whole = tb.compare(gcn, dev, src, dst, 9000, what="hubs, folded grid")
    tb.compare(gcn, dev, src, dst, 9000, 2000, 6500, deg_global=whole.deg, what="hub block, folded grid")
    rng = np.random.default_rng(4)
    s = rng.integers(0, 30000, 400000); d = rng.integers(0, 30000, 400000)
    tb.compare(gcn, dev, s, d, 30000, what="directed, folded grid")


@pytest.fixture(scope="module")
def hub_block(gcn, dev):
    import paper_2212_05009_amd as g
    g.gcn_debug_max_grid_x(CAP)
    src, dst = hub_graph(9000, 3, 6.0, seed=11)
    whole = oracle.graph_build(src, dst, 9000)
    out = tparts.build_both(gcn, dev, src, dst, 9000, 0, 3000, deg_global=whole.deg)
    g.gcn_debug_max_grid_x(0)
    return out


@pytest.mark.parametrize("d", [1, 16, 47, 128, 256, 602])
def test_sparse_products_folded(gcn, dev, hub_block, d):
    og, A = hub_block
    assert og.deg.max() > 2048 and og.nh > 0
    # more blocks than one grid row at every width (the narrow widths pack up to 16 rows into a wavefront)
    tparts.run_parts(gcn, dev, og, A, d, epilogue="relu", bias=True)
    tparts.run_parts(gcn, dev, og, A, d, bf16=True)
    import torch
    rng = np.random.default_rng(d)
    G = rng.standard_normal((og.nr, d)).astype(np.float32)
    ref, bound = oracle.spmm(og.colptr, og.rowidx, og.val_t, G)
    D = torch.full((og.nc, d), float("nan"), device=dev)
    say(f"spmm_t folded rows={og.nc} d={d}")
    gcn.gcn_spmm_t(A, to_dev(G, dev), D)
    torch.cuda.synchronize()
    check_bound(to_np(D), ref, bound, TOL_F32, "A^T G")


@pytest.mark.parametrize("d_in,d_out", [(128, 41), (16, 128), (100, 47)])
def test_layer_folded(gcn, dev, d_in, d_out):
    src, dst = hub_graph(9000, 3, 6.0, seed=5)
    case = tl.Case(gcn, dev, src, dst, 9000)
    tl.run_fwd(gcn, dev, case, d_in, d_out, bias=True, save_ah=True)
    tl.run_bwd(gcn, dev, case, d_in, d_out, dbias=True)          # pads the rows of G where d_out is odd
    tl.run_bwd(gcn, dev, case, d_in, d_out, bf16=True)


@pytest.mark.parametrize("d,bf16", [(33, False), (128, False), (7, True), (300, False)])
def test_gather_folded(gcn, dev, d, bf16):
    import torch
    rng = np.random.default_rng(d)
    nt, n_idx = 5000, 70001
    table = rng.standard_normal((nt, d)).astype(np.float32)
    idx = rng.integers(0, nt, n_idx).astype(np.int32)
    t = to_dev(table, dev).to(torch.bfloat16) if bf16 else to_dev(table, dev)
    want = oracle.gather(to_np(t), idx)
    recv = torch.full((n_idx, d), float("nan"), dtype=t.dtype, device=dev)
    say(f"gather folded n_idx={n_idx} d={d} bf16={bf16}")
    gcn.gcn_halo_gather(t, torch.from_numpy(idx).to(dev), recv)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(recv).view(np.int32), np.asarray(want, np.float32).view(np.int32))


def test_sgd_update_folded(gcn, dev):
    import torch
    rng = np.random.default_rng(9)
    W = rng.standard_normal((1000, 103)).astype(np.float32); dW = rng.standard_normal((1000, 103)).astype(np.float32)
    want = oracle.sgd_update(W, dW, 0.25)
    Wd = to_dev(W, dev)
    gcn.gcn_sgd_update(Wd, to_dev(dW, dev), 0.25)
    torch.cuda.synchronize()
    lim = 1e-6 * (np.abs(W) + np.abs(0.25 * dW))
    assert np.all(np.abs(to_np(Wd).astype(np.float64) - want) <= lim)


def test_induced_and_partition_folded(gcn, dev):
    rng = np.random.default_rng(13)
    n, m = 30000, 400000
    src = rng.integers(0, n, m); dst = rng.integers(0, n, m)
    part = rng.integers(0, 64, n)
    og, A, _ = tp.both(gcn, dev, src, dst, n, part, 64)
    V = rng.permutation(n)[:12000]
    ti.check_induced(gcn, dev, A, src, dst, n, V)


def test_too_large_for_the_cap_is_an_error(gcn, dev):
    """With a cap of 1 a launch holds at most 65535 blocks: a longer index list is refused, not truncated."""
    import torch
    gcn.gcn_debug_max_grid_x(1)
    n_idx = 65535 * 64 + 64 + 1                       # 4-byte rows: 64 rows per block
    table = torch.zeros((8, 1), device=dev)
    idx = torch.zeros(n_idx, dtype=torch.int32, device=dev)
    recv = torch.empty((n_idx, 1), device=dev)
    gcn.gcn_halo_gather(table, idx[:65535 * 4], recv[:65535 * 4])      # fits whatever the rows per block
    with pytest.raises(gcn.GcnError):
        gcn.gcn_halo_gather(table, idx, recv)
