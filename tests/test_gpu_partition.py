"""GPU parity: gcn_partition_stats against the oracle's net-by-net count (Sec. 4.3.2 column-net model, Sec. 5
communication metrics).  Integer work: every figure must be equal."""
import os

import numpy as np
import pytest

import oracle
from util import say

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
KEYS = ("load", "send_rows", "recv_rows", "send_msgs", "recv_msgs")


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def both(gcn, dev, src, dst, n, part, p):
    import torch
    og = oracle.graph_build(src, dst, n)
    A = gcn.gcn_csr_build(torch.from_numpy(np.ascontiguousarray(src, np.int32)).to(dev),
                          torch.from_numpy(np.ascontiguousarray(dst, np.int32)).to(dev), n, 0, n)
    want = oracle.partition_stats(og.colptr, og.rowidx, og.rowptr, part, p)
    say(f"partition_stats n={n} nnz={og.nnz} p={p}")
    got = gcn.gcn_partition_stats(A, torch.from_numpy(np.ascontiguousarray(part, np.int32)).to(dev), p)
    torch.cuda.synchronize()
    for k in KEYS:
        assert got[k].cpu().numpy().tolist() == want[k].tolist(), k
    assert got["totals"].cpu().numpy().tolist() == [want["volume"], want["cut_entries"]]
    return og, A, want


def test_paper_example(gcn, dev):
    facts = {}
    for line in open(os.path.join(GOLDEN, "halo_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, *rest = line.split()
            facts[k] = rest
    e = np.array([[int(x) for x in q.split("-")] for q in facts["edges"]]) - 1
    src = np.concatenate([e[:, 0], e[:, 1]]); dst = np.concatenate([e[:, 1], e[:, 0]])
    part = np.zeros(6, int)
    for m, q in enumerate(facts["parts"]):
        part[[int(x) - 1 for x in q.split(",")]] = m
    _, _, want = both(gcn, dev, src, dst, 6, part, 3)
    assert want["recv_rows"][2] == 3 and want["send_rows"][1] == int(facts["transfers_row4"][0])


@pytest.mark.parametrize("n,m,p,directed,seed", [
    (50, 200, 1, False, 1), (500, 3000, 2, True, 2), (5000, 60000, 7, True, 3), (20000, 300000, 64, False, 4),
    (20000, 150000, 1000, True, 5), (3000, 20000, 3000, False, 6), (70000, 900000, 16, True, 7)])
def test_random_partitions(gcn, dev, n, m, p, directed, seed):
    rng = np.random.default_rng(seed)
    u = rng.integers(0, n, m); v = (u + rng.geometric(0.01, m)) % n if seed % 2 else rng.integers(0, n, m)
    src, dst = (u, v) if directed else (np.r_[u, v], np.r_[v, u])
    part = rng.integers(0, max(1, p - p // 8), n)               # the last eighth of the parts stays empty
    if p == n:
        part = rng.permutation(n)                               # every vertex its own part
    both(gcn, dev, src, dst, n, part, p)


def test_contiguous_parts_match_block_builds(gcn, dev):
    """The rows a contiguous part receives are the halo list of its block build, bit for bit in size."""
    import torch
    rng = np.random.default_rng(9)
    n, m = 30000, 400000
    u = rng.integers(0, n, m); v = (u + rng.geometric(0.002, m)) % n
    src, dst = np.r_[u, v], np.r_[v, u]
    cuts = [0, 5000, 5001, 17000, 30000]
    part = np.zeros(n, int)
    for k in range(4):
        part[cuts[k]:cuts[k + 1]] = k
    og, A, want = both(gcn, dev, src, dst, n, part, 4)
    sd, dd = torch.from_numpy(src.astype(np.int32)).to(dev), torch.from_numpy(dst.astype(np.int32)).to(dev)
    dg = torch.from_numpy(og.deg).to(dev)
    for k in range(4):
        B = gcn.gcn_csr_build(sd, dd, n, cuts[k], cuts[k + 1], deg_global=dg)
        assert (B.nh, B.nnz) == (int(want["recv_rows"][k]), int(want["load"][k]))


def test_config2_random_and_contiguous_partitions(gcn, dev):
    """The bench graph (R-MAT, 2^18 vertices), 8 parts: a random partition against contiguous ranges."""
    from workloads import configs
    w = configs.get("c2_rmat18")
    n = w["n"]
    rng = np.random.default_rng(1)
    _, _, rnd = both(gcn, dev, w["src"], w["dst"], n, rng.integers(0, 8, n), 8)
    assert rnd["volume"] <= rnd["cut_entries"] and rnd["send_rows"].sum() == rnd["recv_rows"].sum() == rnd["volume"]
    assert rnd["send_msgs"].tolist() == [7] * 8


def test_argument_errors(gcn, dev):
    import torch
    rng = np.random.default_rng(2)
    n = 100
    src = torch.from_numpy(rng.integers(0, n, 400).astype(np.int32)).to(dev)
    dst = torch.from_numpy(rng.integers(0, n, 400).astype(np.int32)).to(dev)
    A = gcn.gcn_csr_build(src, dst, n, 0, n)
    part = torch.zeros(n, dtype=torch.int32, device=dev)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_partition_stats(A, part, 0)
    part[17] = 3
    with pytest.raises(gcn.GcnError):
        gcn.gcn_partition_stats(A, part, 3)                     # part id 3 with p = 3
    part[17] = -1
    with pytest.raises(gcn.GcnError):
        gcn.gcn_partition_stats(A, part, 3)
    with pytest.raises(TypeError):
        gcn.gcn_partition_stats(A, part[:-1], 3)
    whole_deg = A.arrays()["deg"]
    B = gcn.gcn_csr_build(src, dst, n, 10, 60, deg_global=whole_deg)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_partition_stats(B, torch.zeros(50, dtype=torch.int32, device=dev), 2)
