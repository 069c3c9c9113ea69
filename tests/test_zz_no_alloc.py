"""GPU test of gcn_spmm_noalloc, the sparse product for callers that cannot allocate: through the C ABI, its
output against gcn_spmm's on two calls in a row, the second on a smaller graph (the fixed scratch array then
still holds the first call's partial rows), with long rows that use that scratch; every output also against
the oracle at 1e-5 * sum|terms|.  Plus the size limit: a matrix whose long-row partials exceed the fixed
buffer is refused with an error and nothing is enqueued.
"""
import numpy as np
import pytest

import oracle
from util import TOL_F32, check_bound, hub_graph, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def _one(gcn, dev, n, n_hubs, d, seed, epilogue):
    import torch
    src, dst = hub_graph(n, n_hubs, 12.0, seed)
    og = oracle.graph_build(src, dst, n)
    assert og.deg.max() > 2048, "no row long enough to use the scratch array"
    A = gcn.gcn_csr_build(torch.from_numpy(src).to(dev), torch.from_numpy(dst).to(dev), n)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d)).astype(np.float32)
    Zp = rng.standard_normal((n, d)).astype(np.float32)
    bias = rng.standard_normal(d).astype(np.float32) if epilogue == gcn.EPI_RELU else None
    Xd = torch.from_numpy(X).to(dev); Zd = torch.from_numpy(Zp).to(dev)
    bd = torch.from_numpy(bias).to(dev) if bias is not None else None
    Y0 = torch.full((n, d), 7.0, device=dev); Y1 = torch.full((n, d), -7.0, device=dev)
    kw = dict(epilogue=epilogue, bias=bd, Zprev=Zd if epilogue == gcn.EPI_MASK else None)
    say(f"gcn_spmm / gcn_spmm_noalloc n={n} hubs={n_hubs} d={d} epilogue={epilogue}")
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", 0)          # the entry point under test never takes the column sweep
    try:
        gcn.gcn_spmm(A, Xd, Y0, **kw)
    finally:
        gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", None)
    gcn.gcn_spmm_noalloc(A, Xd, Y1, **kw)
    torch.cuda.synchronize()
    want, bound = oracle.spmm(og.rowptr, og.col, og.val, X)
    if bias is not None:
        want = want + bias.astype(np.float64); bound = bound + np.abs(bias.astype(np.float64))
    if epilogue == gcn.EPI_RELU:
        want = np.maximum(want, 0.0)
    elif epilogue == gcn.EPI_MASK:
        want = np.where(Zp > 0, want, 0.0)
    y0, y1 = Y0.cpu().numpy(), Y1.cpu().numpy()
    check_bound(y1, want, bound, TOL_F32, f"gcn_spmm_noalloc n={n} d={d}")
    check_bound(y0, want, bound, TOL_F32, f"gcn_spmm n={n} d={d}")
    assert np.array_equal(y0, y1), "the two entry points run the same kernels: results must be identical"
    A.free()


def test_noalloc_matches_spmm_on_two_calls_in_a_row(gcn, dev):
    _one(gcn, dev, n=30000, n_hubs=6, d=96, seed=1, epilogue=gcn.EPI_NONE)
    _one(gcn, dev, n=9000, n_hubs=3, d=40, seed=2, epilogue=gcn.EPI_RELU)       # smaller: stale partial rows beyond it
    _one(gcn, dev, n=12000, n_hubs=4, d=128, seed=3, epilogue=gcn.EPI_MASK)


def test_noalloc_refuses_what_does_not_fit(gcn, dev):
    import torch
    # 80 rows linked to all 300 000 vertices: 80 * 293 chunks of 1024 entries; at 768 features their partial rows
    # would take 72 MB, more than the 64 MiB the fixed array holds
    n, hubs, d = 300_000, 80, 768
    u = np.repeat(np.arange(hubs, dtype=np.int64), n); v = np.tile(np.arange(n, dtype=np.int64), hubs)
    src = np.concatenate([u, v]).astype(np.int32); dst = np.concatenate([v, u]).astype(np.int32)
    A = gcn.gcn_csr_build(torch.from_numpy(src).to(dev), torch.from_numpy(dst).to(dev), n)
    X = torch.zeros(n, d, device=dev); Y = torch.full((n, d), 3.0, device=dev)
    say("gcn_spmm_noalloc beyond its scratch limit")
    with pytest.raises(gcn.GcnError, match="scratch"):
        gcn.gcn_spmm_noalloc(A, X, Y)
    torch.cuda.synchronize()
    assert float(Y.min()) == 3.0 and float(Y.max()) == 3.0        # nothing was enqueued
    gcn.gcn_spmm_noalloc(A, X[:, :512], Y[:, :512])             # 48 MB of partial rows: fits
    torch.cuda.synchronize()
    assert float(Y[:, :512].abs().max()) == 0.0
    A.free()
