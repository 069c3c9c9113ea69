"""GPU parity: the backward pass of one layer in the pull form of Algorithm 2 (Sec. 4.2) against the oracle.

T = A^_m [G_m; G_halo], dH = (T W^T) (.) [Zprev > 0], dW = H_m^T T, dbias = column sums of G_m.  Every
element within 1e-5 * (sum of the absolute values of its terms) in fp32, 2e-2 * the same for bf16 features
(the bf16 path stores T rounded to bf16 before the dense products: 2^-9 relative, inside that bound).
Also in two phases: owned columns first, with NaN in the halo rows of G, then the halo columns and the rest.
"""
import numpy as np
import pytest

import oracle
from util import TOL_BF16, TOL_F32, bf16_round, check_bound, hub_graph, say, to_dev, to_np

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


def build_both(gcn, dev, src, dst, n, lo, hi, deg_global=None):
    import torch
    og = oracle.graph_build(src, dst, n, lo, hi, deg_global=deg_global)
    dg = None if deg_global is None else torch.from_numpy(np.ascontiguousarray(deg_global, np.int32)).to(dev)
    A = gcn.gcn_csr_build(torch.from_numpy(np.ascontiguousarray(src, np.int32)).to(dev),
                          torch.from_numpy(np.ascontiguousarray(dst, np.int32)).to(dev), n, lo, hi, deg_global=dg)
    return og, A


@pytest.fixture(scope="module")
def block(gcn, dev):
    rng = np.random.default_rng(31)
    n, m = 7000, 110000
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    src, dst = np.r_[u, v], np.r_[v, u]
    whole = oracle.graph_build(src, dst, n)
    return build_both(gcn, dev, src, dst, n, 1500, 4321, deg_global=whole.deg)


@pytest.fixture(scope="module")
def hub_block(gcn, dev):
    src, dst = hub_graph(9000, 3, 6.0, seed=13)
    whole = oracle.graph_build(src, dst, 9000)
    return build_both(gcn, dev, src, dst, 9000, 0, 2500, deg_global=whole.deg)


@pytest.fixture(scope="module")
def whole_graph(gcn, dev):
    rng = np.random.default_rng(37)
    n, m = 3000, 30000
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    return build_both(gcn, dev, np.r_[u, v], np.r_[v, u], n, 0, n)


def run_pull(gcn, dev, og, A, d_in, d_out, bf16=False, mask=True, want_dH=True, want_dbias=False, phases=False, seed=0):
    import torch
    rng = np.random.default_rng(900 + seed + 7 * d_in + d_out)
    H = rng.standard_normal((og.nc, d_in)).astype(np.float32)        # only the owned rows are read
    G = rng.standard_normal((og.nc, d_out)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    Zp = rng.standard_normal((og.nr, d_in)).astype(np.float32) if mask else None
    if bf16:
        H, G = bf16_round(H), bf16_round(G)
        Zp = None if Zp is None else bf16_round(Zp)
    ref = oracle.layer_bwd_pull(og, H[: og.nr], W, G, Zprev=Zp)
    tol = TOL_BF16 if bf16 else TOL_F32
    tdt = torch.bfloat16 if bf16 else torch.float32
    Hd, Gd, Wd = to_dev(H, dev, bf16), to_dev(G, dev, bf16), to_dev(W, dev)
    Zd = None if Zp is None else to_dev(Zp, dev, bf16)
    T = torch.full((og.nr, d_out), float("nan"), dtype=tdt, device=dev)
    dH = torch.full((og.nr, d_in), float("nan"), dtype=tdt, device=dev) if want_dH else None
    dW = torch.full((d_in, d_out), float("nan"), device=dev)
    db = torch.full((d_out,), float("nan"), device=dev) if want_dbias else None
    say(f"bwd_pull rows={og.nr} halo={og.nh} {d_in}->{d_out} bf16={bf16} mask={mask} dH={want_dH} phases={phases}")
    if phases:
        Gl = Gd.clone(); Gl[og.nr:] = float("nan")                   # the halo rows have not arrived yet
        gcn.gcn_layer_bwd_pull(A, Hd, Wd, Gl, T, dW, phase=gcn.PART_LOCAL)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(T.float()).all()) and bool(torch.isnan(dW).all())
        gcn.gcn_layer_bwd_pull(A, Hd[: og.nr], Wd, Gd, T, dW, dH=dH, Zprev=Zd, dbias=db, phase=gcn.PART_HALO)
    else:
        gcn.gcn_layer_bwd_pull(A, Hd, Wd, Gd, T, dW, dH=dH, Zprev=Zd, dbias=db)
    torch.cuda.synchronize()
    check_bound(to_np(T), ref["T"], ref["BT"], tol, "T")
    check_bound(to_np(dW), ref["dW"], ref["BdW"], tol, "dW")
    if want_dH:
        check_bound(to_np(dH), ref["dH"], ref["BdH"], tol, "dH")
        if mask:
            assert bool((dH[to_dev(Zp, dev, bf16) <= 0] == 0).all())
    if want_dbias:
        g64 = G[: og.nr].astype(np.float64)
        check_bound(to_np(db), g64.sum(0), np.abs(g64).sum(0), tol, "dbias")


@pytest.mark.parametrize("d_in,d_out", [(128, 128), (128, 16), (16, 41), (100, 47), (602, 128), (5, 3), (64, 256)])
def test_pull_shapes_fp32(gcn, dev, block, d_in, d_out):
    og, A = block
    assert og.nh > 0
    run_pull(gcn, dev, og, A, d_in, d_out, want_dbias=True)


@pytest.mark.parametrize("d_in,d_out", [(128, 128), (128, 16), (100, 47), (64, 256)])
def test_pull_shapes_bf16(gcn, dev, block, d_in, d_out):
    og, A = block
    run_pull(gcn, dev, og, A, d_in, d_out, bf16=True)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d_in,d_out", [(128, 32), (41, 16), (16, 130)])
def test_pull_two_phases(gcn, dev, block, d_in, d_out, bf16):
    og, A = block
    run_pull(gcn, dev, og, A, d_in, d_out, bf16=bf16, phases=True, want_dbias=True)


def test_pull_variants(gcn, dev, block):
    og, A = block
    run_pull(gcn, dev, og, A, 64, 32, mask=False)
    run_pull(gcn, dev, og, A, 64, 32, want_dH=False)
    run_pull(gcn, dev, og, A, 64, 32, want_dH=False, phases=True)


@pytest.mark.parametrize("d_in,d_out", [(47, 128), (128, 16)])
def test_pull_hub_rows(gcn, dev, hub_block, d_in, d_out):
    og, A = hub_block
    assert og.deg.max() > 2048 and og.nh > 0
    run_pull(gcn, dev, og, A, d_in, d_out)
    run_pull(gcn, dev, og, A, d_in, d_out, phases=True, bf16=True)


def test_pull_whole_graph_equals_push_form(gcn, dev, whole_graph):
    """No halo: both phases still work, and on a symmetric graph the result is gcn_layer_bwd's (same oracle bound)."""
    import torch
    og, A = whole_graph
    assert og.nh == 0
    run_pull(gcn, dev, og, A, 64, 16, phases=True)
    rng = np.random.default_rng(3)
    H = rng.standard_normal((og.nc, 64)).astype(np.float32)
    G = rng.standard_normal((og.nr, 16)).astype(np.float32)
    W = rng.standard_normal((64, 16)).astype(np.float32)
    Zp = rng.standard_normal((og.nr, 64)).astype(np.float32)
    ref = oracle.layer_bwd(og, H, W, G, Zprev=Zp)
    T = torch.empty(og.nr, 16, device=dev); dH = torch.empty(og.nr, 64, device=dev); dW = torch.empty(64, 16, device=dev)
    gcn.gcn_layer_bwd_pull(A, to_dev(H, dev), to_dev(W, dev), to_dev(G, dev), T, dW, dH=dH, Zprev=to_dev(Zp, dev))
    torch.cuda.synchronize()
    check_bound(to_np(dW), ref["dW"], ref["BdW"], TOL_F32, "dW vs push form")
    check_bound(to_np(dH), ref["dH"], ref["BdH"], TOL_F32, "dH vs push form")


def test_pull_argument_errors(gcn, dev, block):
    import torch
    og, A = block
    H = torch.zeros(og.nc, 8, device=dev); G = torch.zeros(og.nc, 4, device=dev); W = torch.zeros(8, 4, device=dev)
    T = torch.zeros(og.nr, 4, device=dev); dW = torch.zeros(8, 4, device=dev)
    with pytest.raises(gcn.GcnError):
        gcn.gcn_layer_bwd_pull(A, H, W, G, T, dW, phase=5)
    with pytest.raises(TypeError):
        gcn.gcn_layer_bwd_pull(A, H, W, G[: og.nr], T, dW)
    with pytest.raises(TypeError):
        gcn.gcn_layer_bwd_pull(A, H, W, G, T[:-1], dW)
