"""GPU parity: gcn_csr_build (CSR, CSC, degrees, halo list, values) against the oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from util import hub_graph, say

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


def _dev_i32(a, dev):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)


def compare(gcn, dev, src, dst, n, lo=0, hi=None, deg_global=None, what=""):
    hi = n if hi is None else hi
    say(f"csr_build {what} n={n} E={len(src)} block=[{lo},{hi})")
    og = oracle.graph_build(src, dst, n, lo, hi, deg_global=deg_global)
    dg = None if deg_global is None else _dev_i32(deg_global, dev)
    A = gcn.gcn_csr_build(_dev_i32(src, dev), _dev_i32(dst, dev), n, lo, hi, deg_global=dg)
    assert (A.nr, A.nh, A.nnz) == (og.nr, og.nh, og.nnz)
    arr = {k: (None if v is None else v.cpu().numpy()) for k, v in A.arrays().items()}
    for name in ["rowptr", "col", "deg", "halo_gid", "colptr", "rowidx"]:
        assert np.array_equal(arr[name], getattr(og, name)), f"{what}: {name} differs"
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].view(np.int32), getattr(og, name).view(np.int32)), f"{what}: {name} differs"
    A.free()
    return og


def test_build_config1(gcn, dev, c1):
    compare(gcn, dev, c1["src"], c1["dst"], c1["n"], what="c1")


def test_build_paper_halo_example(gcn, dev):
    # Sec. 4.1 worked example: processor 3 owns v5, v6 and receives rows {1, 2} and {4}
    e = np.array([[1, 2], [1, 5], [2, 4], [2, 6], [3, 4], [4, 5], [4, 6]]) - 1
    src = np.concatenate([e[:, 0], e[:, 1]]); dst = np.concatenate([e[:, 1], e[:, 0]])
    whole = compare(gcn, dev, src, dst, 6, what="example whole")
    og = compare(gcn, dev, src, dst, 6, 4, 6, deg_global=whole.deg, what="example block")
    assert og.halo_gid.tolist() == [0, 1, 3]


@pytest.mark.parametrize("seed,directed", [(1, False), (2, True)])
def test_build_random_blocks(gcn, dev, seed, directed):
    rng = np.random.default_rng(seed)
    n, m = 5000, 60000
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    if directed:
        src, dst = u, v
    else:
        src, dst = np.concatenate([u, v]), np.concatenate([v, u])
    whole = compare(gcn, dev, src, dst, n, what=f"random seed={seed}")
    for lo, hi in [(0, 1), (0, 1700), (1700, 1701), (1701, 4999), (4999, 5000)]:
        compare(gcn, dev, src, dst, n, lo, hi, deg_global=whole.deg, what=f"random seed={seed} block")


def test_build_duplicates_self_loops_isolated(gcn, dev):
    # heavy duplication, self-loops, vertices with no edge at all (rows holding only the diagonal)
    rng = np.random.default_rng(3)
    n = 700
    u = rng.integers(0, 40, 30000); v = rng.integers(0, 40, 30000)
    src = np.concatenate([u, v, np.arange(50)]); dst = np.concatenate([v, u, np.arange(50)])
    og = compare(gcn, dev, src, dst, n, what="duplicates")
    assert og.nnz < 40 * 40 + n + 1 and np.all(og.deg[40:] == 1)
    compare(gcn, dev, np.zeros(0, np.int32), np.zeros(0, np.int32), 5, what="no edges")
    compare(gcn, dev, [0], [0], 1, what="single vertex")


def test_build_hub_rows(gcn, dev):
    src, dst = hub_graph(9000, 3, 6.0, seed=5)
    og = compare(gcn, dev, src, dst, 9000, what="hubs")
    assert og.deg.max() >= 9000 - 1
    whole_deg = og.deg
    compare(gcn, dev, src, dst, 9000, 0, 100, deg_global=whole_deg, what="hub block")


def test_build_rejects_bad_input(gcn, dev):
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_build(_dev_i32([0, 7], dev), _dev_i32([1, 2], dev), 4)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_build(_dev_i32([0, -1], dev), _dev_i32([1, 2], dev), 4)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_build(_dev_i32([0], dev), _dev_i32([1], dev), 4, 0, 2)       # block without global degrees
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_build(_dev_i32([0], dev), _dev_i32([1], dev), 4, 0, 2, deg_global=_dev_i32([1, 0, 1, 1], dev))
    with pytest.raises(gcn.GcnError):
        gcn.gcn_csr_build(_dev_i32([0], dev), _dev_i32([1], dev), 4, 3, 2)
    # without CSC the transpose is refused, not run
    import torch
    A = gcn.gcn_csr_build(_dev_i32([0, 1], dev), _dev_i32([1, 0], dev), 2, flags=0)
    assert A.arrays()["colptr"] is None
    X = torch.zeros(2, 4, device=dev); Y = torch.zeros(2, 4, device=dev)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_spmm_t(A, X, Y)
    A.free()
