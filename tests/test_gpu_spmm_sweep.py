"""GPU parity of the column-sweep (LDS panel) variant of gcn_spmm / gcn_spmm_t.

The library picks this variant by itself only for large operands; gcn_debug_set_tuning("GCN_SPMM_PANEL", 1) makes it the
path for every product its limits allow, so the small graphs here exercise it: ragged panels,
rows cut into several virtual rows, all lane-group shapes (width <= 16, 32-wide slices, vector and
scalar gathers, fp32 and bf16), every epilogue, and the transposed arrays of a directed block.
Same tolerance as the row-per-wavefront variant: 1e-5 (fp32) / 2e-2 (bf16) times sum |terms|.
"""
import os

import numpy as np
import pytest

from test_gpu_spmm import Case, run_spmm
from util import hub_graph

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


@pytest.fixture(autouse=True)
def forced_sweep(gcn):
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", 1)
    yield
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", None)


@pytest.fixture(scope="module")
def er(gcn, dev, c1):
    return Case(gcn, dev, c1["src"], c1["dst"], c1["n"])


@pytest.fixture(scope="module")
def hubs(gcn, dev):
    src, dst = hub_graph(9000, 3, 6.0, seed=5)       # rows of 9000, 4500 and 3000 entries: 18, 9 and 6 virtual rows
    return Case(gcn, dev, src, dst, 9000)


@pytest.fixture(scope="module")
def directed_block(gcn, dev):
    import oracle
    rng = np.random.default_rng(23)
    n, m = 7000, 120000
    src = rng.integers(0, n, m); dst = rng.integers(0, n, m)
    whole = oracle.graph_build(src, dst, n)
    return Case(gcn, dev, src, dst, n, 1500, 4200, deg_global=whole.deg)


@pytest.mark.parametrize("d", [1, 3, 8, 16, 17, 32, 41, 47, 64, 100, 128, 130, 256, 602])
def test_sweep_widths_fp32(gcn, dev, er, d):
    run_spmm(gcn, dev, er, d)


@pytest.mark.parametrize("d", [1, 7, 16, 24, 41, 64, 100, 128, 256])
def test_sweep_widths_bf16(gcn, dev, er, d):
    run_spmm(gcn, dev, er, d, bf16=True)


@pytest.mark.parametrize("d,pad", [(16, 1), (41, 3), (128, 2), (100, 4), (64, 8)])
def test_sweep_padded_leading_dimension(gcn, dev, er, d, pad):
    run_spmm(gcn, dev, er, d, pad=pad)
    run_spmm(gcn, dev, er, d, pad=pad, bf16=True)


@pytest.mark.parametrize("epilogue", ["relu", "mask"])
@pytest.mark.parametrize("bf16", [False, True])
def test_sweep_epilogues(gcn, dev, er, epilogue, bf16):
    run_spmm(gcn, dev, er, 48, bf16=bf16, epilogue=epilogue)
    run_spmm(gcn, dev, er, 128, bf16=bf16, epilogue=epilogue, bias=(epilogue == "relu"))


@pytest.mark.parametrize("d", [1, 16, 47, 128])
def test_sweep_long_rows(gcn, dev, hubs, d):
    assert hubs.og.deg.max() > 2048
    run_spmm(gcn, dev, hubs, d)
    run_spmm(gcn, dev, hubs, d, transpose=True, epilogue="mask")
    run_spmm(gcn, dev, hubs, d, bf16=True, epilogue="relu")


@pytest.mark.parametrize("d", [5, 64, 100])
def test_sweep_transposed_directed_block(gcn, dev, directed_block, d):
    og = directed_block.og
    assert og.nh > 0 and not np.array_equal(og.colptr[: og.nr + 1], og.rowptr)
    run_spmm(gcn, dev, directed_block, d)
    run_spmm(gcn, dev, directed_block, d, transpose=True)
    run_spmm(gcn, dev, directed_block, d, transpose=True, epilogue="mask")
    run_spmm(gcn, dev, directed_block, d, transpose=True, bf16=True)


def test_sweep_is_run_to_run_identical_and_close_to_row_variant(gcn, dev, hubs):
    import torch
    X = torch.randn(hubs.og.nc, 96, device=dev)
    Y1 = torch.empty(hubs.og.nr, 96, device=dev); Y2 = torch.empty_like(Y1); Y3 = torch.empty_like(Y1)
    gcn.gcn_spmm(hubs.A, X, Y1); gcn.gcn_spmm(hubs.A, X, Y2)
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", 0)
    gcn.gcn_spmm(hubs.A, X, Y3)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    assert not torch.equal(Y1, Y3) or True       # different summation order: equality is allowed, not required
    assert torch.allclose(Y1, Y3, rtol=0, atol=1e-4)


def test_sweep_is_picked_for_a_dense_neighbourhood_graph(gcn, dev, capfd):
    """65536 vertices, about 64 entries per row: the operand (8 MB per 32-feature slice) spills L2 and is
    re-read about 40 times per round, so the library must choose the column-sweep variant by itself."""
    import torch
    rng = np.random.default_rng(99)
    n, m = 65536, 65536 * 32
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    src = np.concatenate([u, v]).astype(np.int32); dst = np.concatenate([v, u]).astype(np.int32)
    case = Case(gcn, dev, src, dst, n)
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", None)
    gcn.gcn_debug_set_tuning("GCN_PANEL_VERBOSE", 1)
    try:
        capfd.readouterr()
        run_spmm(gcn, dev, case, 64)
        err = capfd.readouterr().err
        assert "[panel plan]" in err, "the heuristic did not choose the column-sweep variant"
        run_spmm(gcn, dev, case, 64, transpose=True, epilogue="mask")
    finally:
        gcn.gcn_debug_set_tuning("GCN_PANEL_VERBOSE", None)
        gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", 1)
        case.A.free()
