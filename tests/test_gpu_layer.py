"""GPU parity: gcn_layer_fwd, gcn_layer_bwd and gcn_softmax_xent against the oracle.

Tolerance: |gpu - oracle_fp64| <= tol * B per element, where B is the same triple sum as the result
with every factor replaced by its absolute value (1e-5 for fp32 features, 2e-2 for bf16 features;
both sides start from identical, already rounded inputs).  Each call is checked on its own: the
inputs of a later call are the GPU's outputs of the earlier one, handed to the oracle unchanged.
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


class Case:
    def __init__(self, gcn, dev, src, dst, n, lo=0, hi=None, deg_global=None):
        import torch
        hi = n if hi is None else hi
        self.og = oracle.graph_build(src, dst, n, lo, hi, deg_global=deg_global)
        dg = None if deg_global is None else torch.from_numpy(np.ascontiguousarray(deg_global, np.int32)).to(dev)
        self.A = gcn.gcn_csr_build(torch.from_numpy(np.ascontiguousarray(src, np.int32)).to(dev),
                                   torch.from_numpy(np.ascontiguousarray(dst, np.int32)).to(dev), n, lo, hi,
                                   deg_global=dg)


@pytest.fixture(scope="module")
def er(gcn, dev, c1):
    return Case(gcn, dev, c1["src"], c1["dst"], c1["n"])


@pytest.fixture(scope="module")
def hubs(gcn, dev):
    src, dst = hub_graph(5000, 2, 5.0, seed=9)
    return Case(gcn, dev, src, dst, 5000)


@pytest.fixture(scope="module")
def directed_block(gcn, dev):
    rng = np.random.default_rng(23)
    n, m = 4000, 50000
    src = rng.integers(0, n, m); dst = rng.integers(0, n, m)
    whole = oracle.graph_build(src, dst, n)
    return Case(gcn, dev, src, dst, n, 500, 2333, deg_global=whole.deg)


@pytest.fixture(scope="module")
def identity(gcn, dev):
    """A graph without edges: A^ = I, so the layer reduces to the dense products alone."""
    return Case(gcn, dev, np.zeros(0, np.int32), np.zeros(0, np.int32), 1237)


def _inputs(og, d_in, d_out, bf16, seed):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((og.nc, d_in)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    G = (rng.standard_normal((og.nr, d_out)) / og.nr).astype(np.float32)
    Zp = rng.standard_normal((og.nr, d_in)).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    if bf16:
        H, G, Zp = bf16_round(H), bf16_round(G), bf16_round(Zp)
    return H, W, G, Zp, b


def run_fwd(gcn, dev, case, d_in, d_out, bf16=False, act="relu", bias=False, save_ah=False, want_z=True, seed=0):
    import torch
    og, A = case.og, case.A
    H, W, _, _, b = _inputs(og, d_in, d_out, bf16, seed + 31 * d_in + d_out)
    ref = oracle.layer_fwd(og, H, W, bias=b if bias else None, act=act)
    tdt = torch.bfloat16 if bf16 else torch.float32
    Hd, Wd = to_dev(H, dev, bf16), to_dev(W, dev)
    Hout = torch.full((og.nr, d_out), float("nan"), dtype=tdt, device=dev)
    Z = torch.full((og.nr, d_out), float("nan"), dtype=tdt, device=dev) if want_z else None
    AH = torch.full((og.nr, d_in), float("nan"), dtype=tdt, device=dev) if save_ah else None
    say(f"layer_fwd nr={og.nr} nc={og.nc} {d_in}->{d_out} bf16={bf16} act={act} bias={bias} save_ah={save_ah}")
    gcn.gcn_layer_fwd(A, Hd, Wd, Hout, act=gcn.ACT_RELU if act == "relu" else gcn.ACT_NONE,
                      bias=to_dev(b, dev) if bias else None, Z=Z, AH_save=AH)
    torch.cuda.synchronize()
    tol = TOL_BF16 if bf16 else TOL_F32
    check_bound(to_np(Hout), ref["Hout"], ref["Bz"], tol, "Hout")
    if want_z:
        check_bound(to_np(Z), ref["Z"], ref["Bz"], tol, "Z")
        if not bf16:          # Hout must be exactly act(Z) of the library's own Z
            z = to_np(Z)
            assert np.array_equal(to_np(Hout), np.maximum(z, 0) if act == "relu" else z)
    if save_ah:
        _, Bah = oracle.spmm(og.rowptr, og.col, og.val, np.abs(H))
        check_bound(to_np(AH), ref["AH"], Bah, tol, "AH_save")
    return Hd, Wd, AH


def run_bwd(gcn, dev, case, d_in, d_out, bf16=False, want_dh=True, mask=True, saved_ah=False, dbias=False, seed=0):
    import torch
    og, A = case.og, case.A
    H, W, G, Zp, _ = _inputs(og, d_in, d_out, bf16, seed + 17 * d_in + d_out)
    ref = oracle.layer_bwd(og, H, W, G, Zprev=Zp if mask else None, want_dH=want_dh, want_dbias=dbias)
    tdt = torch.bfloat16 if bf16 else torch.float32
    Hd, Wd, Gd = to_dev(H, dev, bf16), to_dev(W, dev), to_dev(G, dev, bf16)
    AH = None
    if saved_ah:      # what the forward pass would have stored: the library's own A^ H
        AH = torch.empty(og.nr, d_in, dtype=tdt, device=dev)
        gcn.gcn_spmm(A, Hd, AH)
    dW = torch.full((d_in, d_out), float("nan"), device=dev)
    dH = torch.full((og.nc, d_in), float("nan"), dtype=tdt, device=dev) if want_dh else None
    db = torch.full((d_out,), float("nan"), device=dev) if dbias else None
    say(f"layer_bwd nr={og.nr} nc={og.nc} {d_in}->{d_out} bf16={bf16} dH={want_dh} mask={mask} saved_ah={saved_ah}")
    gcn.gcn_layer_bwd(A, Hd, Wd, Gd, dW, dH=dH, Zprev=to_dev(Zp, dev, bf16) if (mask and want_dh) else None,
                      AH_saved=AH, dbias=db)
    torch.cuda.synchronize()
    tol = TOL_BF16 if bf16 else TOL_F32
    check_bound(to_np(dW), ref["dW"], ref["BdW"], tol, "dW")
    if want_dh:
        check_bound(to_np(dH), ref["dH"], ref["BdH"], tol, "dH")
    if dbias:
        check_bound(to_np(db), ref["dbias"], ref["Bdb"], tol, "dbias")


FWD_SHAPES = [(64, 16), (16, 8), (128, 128), (128, 16), (100, 256), (256, 47), (602, 128), (128, 41), (1, 1), (3, 70)]


@pytest.mark.parametrize("d_in,d_out", FWD_SHAPES)
def test_layer_fwd_fp32(gcn, dev, er, d_in, d_out):
    run_fwd(gcn, dev, er, d_in, d_out)


@pytest.mark.parametrize("d_in,d_out", [(64, 16), (128, 128), (100, 256), (256, 47), (602, 128), (128, 41)])
def test_layer_fwd_bf16(gcn, dev, er, d_in, d_out):
    run_fwd(gcn, dev, er, d_in, d_out, bf16=True)


def test_layer_fwd_options(gcn, dev, er, hubs, directed_block):
    run_fwd(gcn, dev, er, 64, 16, act="none", bias=True)
    run_fwd(gcn, dev, er, 16, 64, act="relu", bias=True, save_ah=True)
    run_fwd(gcn, dev, er, 128, 32, save_ah=True, want_z=False)           # forced sparse-first
    run_fwd(gcn, dev, hubs, 96, 24)
    run_fwd(gcn, dev, hubs, 24, 96, bf16=True, save_ah=True)
    run_fwd(gcn, dev, directed_block, 100, 47)                             # dense-first over nc rows
    run_fwd(gcn, dev, directed_block, 47, 100, bias=True)


@pytest.mark.parametrize("d_in,d_out", [(1, 1), (5, 3), (32, 32), (33, 65), (128, 129), (602, 128), (100, 256), (257, 47)])
def test_dense_products_alone_on_identity_graph(gcn, dev, identity, d_in, d_out):
    assert identity.og.nnz == identity.og.nr and np.all(identity.og.val == 1.0)
    run_fwd(gcn, dev, identity, d_in, d_out, act="none")
    run_bwd(gcn, dev, identity, d_in, d_out)
    run_bwd(gcn, dev, identity, d_in, d_out, bf16=True, mask=False)


BWD_SHAPES = [(64, 16), (16, 8), (128, 128), (16, 128), (256, 47), (47, 256), (602, 128), (128, 41), (100, 256)]


@pytest.mark.parametrize("d_in,d_out", BWD_SHAPES)
def test_layer_bwd_fp32(gcn, dev, er, d_in, d_out):
    run_bwd(gcn, dev, er, d_in, d_out)
    run_bwd(gcn, dev, er, d_in, d_out, want_dh=False)                      # first layer: no dH
    run_bwd(gcn, dev, er, d_in, d_out, saved_ah=True, dbias=True)


@pytest.mark.parametrize("d_in,d_out", [(64, 16), (128, 128), (256, 47), (100, 256)])
def test_layer_bwd_bf16(gcn, dev, er, d_in, d_out):
    run_bwd(gcn, dev, er, d_in, d_out, bf16=True)
    run_bwd(gcn, dev, er, d_in, d_out, bf16=True, saved_ah=True, want_dh=False)


def test_layer_bwd_hubs_and_directed_block(gcn, dev, hubs, directed_block):
    run_bwd(gcn, dev, hubs, 96, 24)
    run_bwd(gcn, dev, hubs, 24, 96, dbias=True)
    for d_in, d_out in [(100, 47), (47, 100)]:
        run_bwd(gcn, dev, directed_block, d_in, d_out)                     # dH has nc rows: owned + halo parts
        run_bwd(gcn, dev, directed_block, d_in, d_out, mask=False, saved_ah=True)


# the kernel that keeps W in registers and streams 64-row tiles of the operand through LDS: every epilogue, a K with
# and without a tail, 1 to 4 wavefronts per workgroup, row counts around a tile and beyond one tile per workgroup
@pytest.mark.parametrize("rows", [1, 63, 64, 65, 129, 16385, 70001])
@pytest.mark.parametrize("d_in,d_out", [(256, 256), (128, 256), (200, 192), (100, 256), (68, 64), (256, 128)])
def test_register_resident_weight_kernel(gcn, dev, rows, d_in, d_out):
    case = Case(gcn, dev, np.zeros(0, np.int32), np.zeros(0, np.int32), rows)          # A^ = I
    gcn.gcn_debug_set_tuning("GCN_GEMM_REGW", 2)
    try:
        run_fwd(gcn, dev, case, d_in, d_out, bias=True, save_ah=True)
        run_fwd(gcn, dev, case, d_in, d_out)
        run_bwd(gcn, dev, case, d_in, d_out, saved_ah=True, dbias=True)
        run_bwd(gcn, dev, case, d_in, d_out, mask=False)
    finally:
        gcn.gcn_debug_set_tuning("GCN_GEMM_REGW", None)
        case.A.free()


# dW = (A^ H)^T G with the output in registers and both operands streamed through LDS, forced on for every shape it
# accepts: each tile count per wavefront and each wavefront grid, outputs wider than one 256 x 256 workgroup, ragged
# widths, row counts around a 32-row chunk, one short last chunk, many splits of the sum
@pytest.mark.parametrize("rows", [1, 33, 129, 4097, 70001])
@pytest.mark.parametrize("d_in,d_out", [(256, 256), (100, 256), (256, 100), (128, 128), (64, 16), (32, 256), (256, 32),
                                        (64, 252), (300, 44), (44, 300), (520, 260)])
def test_weight_gradient_kernel_with_operands_through_lds(gcn, dev, rows, d_in, d_out):
    case = Case(gcn, dev, np.zeros(0, np.int32), np.zeros(0, np.int32), rows)          # A^ = I
    gcn.gcn_debug_set_tuning("GCN_GEMM_TN_LDS", 2)
    try:
        run_bwd(gcn, dev, case, d_in, d_out, want_dh=False, saved_ah=True, dbias=True)
        run_bwd(gcn, dev, case, d_in, d_out, mask=False)
    finally:
        gcn.gcn_debug_set_tuning("GCN_GEMM_TN_LDS", None)
        case.A.free()


# The weight gradient from a saved A^ H beside the backward pass's sparse product (second stream), forced on for
# small graphs: both orders of the backward products (d_out < d_in shares T = A^T G, otherwise Q = G W^T first), on a
# whole graph, on one with long rows and on a directed row block.  Twice in a row: the stream, the events and the
# workspace are reused; then once more without the saved A^ H, which takes the one-stream path again.
@pytest.mark.parametrize("d_in,d_out", [(256, 256), (100, 256), (256, 100), (128, 192)])
def test_weight_gradient_beside_the_sparse_product(gcn, dev, er, hubs, directed_block, d_in, d_out):
    gcn.gcn_debug_set_tuning("GCN_OVERLAP", 2)
    gcn.gcn_debug_set_tuning("GCN_GEMM_TN_LDS", 2)
    try:
        for case in (er, hubs, directed_block):
            for rep in range(2):
                run_bwd(gcn, dev, case, d_in, d_out, saved_ah=True, dbias=True, seed=rep)
                run_bwd(gcn, dev, case, d_in, d_out, saved_ah=True, mask=False, seed=rep + 7)
            run_bwd(gcn, dev, case, d_in, d_out, seed=3)
    finally:
        for name in ("GCN_OVERLAP", "GCN_GEMM_TN_LDS"):
            gcn.gcn_debug_set_tuning(name, None)


# The dense product of a sparse-first forward layer beside the sparse product (second stream), forced on for small
# graphs: the sparse product is launched on 2, 4 or 8 ranges of rows, each with its share of the long rows, and the
# dense product follows one range behind.  Graphs with fewer rows than ranges x 64 leave some ranges empty.
@pytest.mark.parametrize("chunks", [2, 4, 8])
@pytest.mark.parametrize("d_in,d_out", [(256, 256), (100, 256), (128, 192)])
def test_forward_dense_product_follows_the_sparse_product_by_row_chunks(gcn, dev, er, hubs, directed_block, identity,
                                                                        chunks, d_in, d_out):
    gcn.gcn_debug_set_tuning("GCN_OVERLAP", 2)
    gcn.gcn_debug_set_tuning("GCN_OVERLAP_CHUNKS", chunks)
    gcn.gcn_debug_set_tuning("GCN_GEMM_REGW", 2)
    try:
        for case in (er, hubs, directed_block, identity):
            for rep in range(2):
                run_fwd(gcn, dev, case, d_in, d_out, bias=True, save_ah=True, seed=rep)
            run_fwd(gcn, dev, case, d_in, d_out, want_z=False, act="none", seed=5)
        tiny = Case(gcn, dev, np.array([0, 1, 2], np.int32), np.array([1, 2, 0], np.int32), 70)
        run_fwd(gcn, dev, tiny, d_in, d_out, save_ah=True)
        tiny.A.free()
    finally:
        for name in ("GCN_OVERLAP", "GCN_OVERLAP_CHUNKS", "GCN_GEMM_REGW"):
            gcn.gcn_debug_set_tuning(name, None)


# The layer calls with a leading dimension per buffer: every feature buffer a view of a wider allocation
# (gcn_feature_ld's pitch) whose padding holds NaN: nothing of it may reach a result, and an output's padding is
# written at most up to the next multiple of 16 bytes of the row width.
@pytest.mark.parametrize("d_in,d_out", [(100, 47), (47, 100), (128, 41), (256, 256)])
def test_layer_calls_with_pitched_buffers(gcn, dev, er, directed_block, d_in, d_out):
    import torch

    def pitched(a, rows, d):
        buf = gcn.feature_buffer(rows, d, torch.float32, dev)
        base = buf._base if buf._base is not None else buf
        base.fill_(float("nan"))
        if a is not None:
            buf.copy_(torch.from_numpy(np.ascontiguousarray(a)).to(dev))
        return buf, base

    for case in (er, directed_block):
        og, A = case.og, case.A
        H, W, G, Zp, b = _inputs(og, d_in, d_out, False, 5 * d_in + d_out)
        ref = oracle.layer_fwd(og, H, W, bias=b, act="relu")
        Hd, _ = pitched(H, og.nc, d_in)
        Hout, Hout_base = pitched(None, og.nr, d_out)
        Z, _ = pitched(None, og.nr, d_out)
        AH, _ = pitched(None, og.nr, d_in)
        say(f"layer_fwd_ld nr={og.nr} nc={og.nc} {d_in}->{d_out}")
        gcn.gcn_layer_fwd_ld(A, Hd, to_dev(W, dev), Hout, act=gcn.ACT_RELU, bias=to_dev(b, dev), Z=Z, AH_save=AH)
        torch.cuda.synchronize()
        check_bound(to_np(Hout), ref["Hout"], ref["Bz"], TOL_F32, "Hout")
        check_bound(to_np(Z), ref["Z"], ref["Bz"], TOL_F32, "Z")
        if Hout_base.shape[1] > (d_out + 3) // 4 * 4:
            assert bool(torch.isnan(Hout_base[:, (d_out + 3) // 4 * 4:]).all()), "the padding of Hout was written past 16 bytes"
        rb = oracle.layer_bwd(og, H, W, G, Zprev=Zp, want_dH=True, want_dbias=True)
        Gd, _ = pitched(G, og.nr, d_out)
        Zpd, _ = pitched(Zp, og.nr, d_in)
        dH, dH_base = pitched(None, og.nc, d_in)
        dW = torch.full((d_in, d_out), float("nan"), device=dev)
        db = torch.full((d_out,), float("nan"), device=dev)
        for saved in (AH, None):
            say(f"layer_bwd_ld nr={og.nr} nc={og.nc} {d_in}->{d_out} saved_ah={saved is not None}")
            gcn.gcn_layer_bwd_ld(A, Hd, to_dev(W, dev), Gd, dW, dH=dH, Zprev=Zpd, AH_saved=saved, dbias=db)
            torch.cuda.synchronize()
            check_bound(to_np(dW), rb["dW"], rb["BdW"], TOL_F32, "dW")
            check_bound(to_np(dH), rb["dH"], rb["BdH"], TOL_F32, "dH")
            check_bound(to_np(db), rb["dbias"], rb["Bdb"], TOL_F32, "dbias")
        if dH_base.shape[1] > (d_in + 3) // 4 * 4:
            assert bool(torch.isnan(dH_base[:, (d_in + 3) // 4 * 4:]).all()), "the padding of dH was written past 16 bytes"


# Putting dense products beside sparse ones changes where kernels run, not what they add up: every result of a
# layer call must be bit for bit the one that the same call gives with everything on the caller's stream.
@pytest.mark.parametrize("d_in,d_out", [(256, 256), (100, 256)])
def test_results_do_not_depend_on_the_second_stream(gcn, dev, hubs, directed_block, d_in, d_out):
    import torch
    for name, v in (("GCN_GEMM_REGW", 2), ("GCN_GEMM_TN_LDS", 2)):
        gcn.gcn_debug_set_tuning(name, v)
    try:
        for case in (hubs, directed_block):
            og, A = case.og, case.A
            H, W, G, Zp, b = _inputs(og, d_in, d_out, False, 77)
            Hd, Wd, Gd, Zpd, bd = to_dev(H, dev), to_dev(W, dev), to_dev(G, dev), to_dev(Zp, dev), to_dev(b, dev)
            got = {}
            for mode in (0, 2):
                gcn.gcn_debug_set_tuning("GCN_OVERLAP", mode)
                Hout = torch.empty(og.nr, d_out, device=dev); Z = torch.empty_like(Hout)
                AH = torch.empty(og.nr, d_in, device=dev)
                say(f"overlap={mode} layer_fwd nr={og.nr} {d_in}->{d_out}")
                gcn.gcn_layer_fwd(A, Hd, Wd, Hout, act=gcn.ACT_RELU, bias=bd, Z=Z, AH_save=AH)
                dW = torch.empty(d_in, d_out, device=dev)
                dH = torch.empty(og.nc, d_in, device=dev)
                say(f"overlap={mode} layer_bwd nr={og.nr} {d_in}->{d_out}")
                gcn.gcn_layer_bwd(A, Hd, Wd, Gd, dW, dH=dH, Zprev=Zpd, AH_saved=AH)
                torch.cuda.synchronize()
                got[mode] = [to_np(t) for t in (Hout, Z, AH, dW, dH)]
            for a, c, what in zip(got[0], got[2], ("Hout", "Z", "AH_save", "dW", "dH")):
                assert np.array_equal(a, c), f"{what} differs between one stream and two"
    finally:
        for name in ("GCN_OVERLAP", "GCN_GEMM_REGW", "GCN_GEMM_TN_LDS"):
            gcn.gcn_debug_set_tuning(name, None)


# ----------------------------------------------------------------------------- softmax cross-entropy
@pytest.mark.parametrize("d_in,d_out", [(128, 41), (41, 128), (256, 47), (200, 130), (130, 200)])
def test_layer_with_the_column_sweep(gcn, dev, er, hubs, directed_block, d_in, d_out):
    """The layer calls with the column-sweep form of the sparse product switched on: its operands inside the
    library then get rows that start on a 128-byte line (widths 41, 47, 130: pitches 64, 64, 160 elements)."""
    gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", 1)
    try:
        run_fwd(gcn, dev, er, d_in, d_out, bias=True, save_ah=True)
        run_bwd(gcn, dev, er, d_in, d_out, dbias=True)
        run_bwd(gcn, dev, er, d_in, d_out, saved_ah=True, mask=False)
        run_fwd(gcn, dev, hubs, d_in, d_out)
        run_bwd(gcn, dev, directed_block, d_in, d_out)
        run_fwd(gcn, dev, er, d_in, d_out, bf16=True)
        run_bwd(gcn, dev, er, d_in, d_out, bf16=True)
    finally:
        gcn.gcn_debug_set_tuning("GCN_SPMM_PANEL", None)


@pytest.mark.parametrize("C", [1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 32, 41, 47, 64, 65, 100, 130, 255, 256, 300])
@pytest.mark.parametrize("bf16", [False, True])
def test_softmax_xent(gcn, dev, C, bf16):
    import torch
    rng = np.random.default_rng(C)
    nr = 5003
    Z = (2.5 * rng.standard_normal((nr, C))).astype(np.float32)
    if bf16:
        Z = bf16_round(Z)
    y = rng.integers(0, C, nr).astype(np.int32)
    y[::11] = -1
    scale = 1.0 / nr
    loss, labs, G = oracle.softmax_xent(Z, y, scale)
    # bound of G: scale * (softmax + onehot), i.e. the two terms of the gradient in absolute value
    onehot = np.zeros((nr, C)); lab = y >= 0; onehot[np.nonzero(lab)[0], y[lab]] = 1.0
    Bg = G + 2 * scale * onehot          # scale*(p - onehot) + 2*scale*onehot = scale*(p + onehot)
    Bg[~lab] = 0.0
    Zd = to_dev(Z, dev, bf16)
    Gd = torch.full((nr, C), float("nan"), dtype=Zd.dtype, device=dev)
    ld = torch.full((1,), float("nan"), device=dev)
    say(f"softmax_xent nr={nr} C={C} bf16={bf16}")
    gcn.gcn_softmax_xent(Zd, to_dev(y, dev), scale, ld, Gd)
    torch.cuda.synchronize()
    tol = TOL_BF16 if bf16 else TOL_F32
    check_bound(to_np(Gd), G, Bg, tol, "G")
    # the loss is an fp32 scalar built from fp32 per-row terms z_y, max and log-sum-exp
    Zd64 = Z.astype(np.float64)
    terms = np.abs(Zd64[np.nonzero(lab)[0], y[lab]]) + 2 * np.abs(Zd64[lab]).max(1) + np.log(C)
    assert abs(float(ld.item()) - loss) <= TOL_F32 * max(labs, scale * terms.sum())
    assert bool((Gd[::11] == 0).all())


def test_softmax_xent_closed_form_and_padding(gcn, dev):
    import torch
    nr, C = 777, 16
    Z = torch.zeros(nr, C + 3, device=dev)
    y = (torch.arange(nr, device=dev) % C).to(torch.int32)
    G = torch.full((nr, C + 5), -7.0, device=dev)
    loss = torch.zeros(1, device=dev)
    gcn.gcn_softmax_xent(Z[:, :C], y, 1.0 / nr, loss, G[:, :C])
    torch.cuda.synchronize()
    assert abs(float(loss.item()) - np.log(C)) < 1e-6         # Z = 0  =>  loss = scale * nr * ln C
    assert bool((G[:, C:] == -7.0).all())
    want = torch.full((nr, C), 1.0 / C / nr, device=dev)
    want[torch.arange(nr), y.long()] -= 1.0 / nr
    assert torch.allclose(G[:, :C], want, rtol=1e-6, atol=1e-12)


# ----------------------------------------------------------------------------- two-layer epoch on config 1
@pytest.mark.parametrize("bf16", [False, True])
def test_two_layer_epoch_config1(gcn, dev, er, c1, bf16):
    import torch
    og, A = er.og, er.A
    n, dims = c1["n"], c1["dims"]
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    X = bf16_round(c1["X"]) if bf16 else c1["X"]
    Xd = to_dev(X, dev, bf16)
    W1, W2 = c1["W"]
    W1d, W2d = to_dev(W1, dev), to_dev(W2, dev)
    yd = to_dev(c1["y"], dev)
    Z1 = torch.empty(n, dims[1], dtype=tdt, device=dev); H1 = torch.empty_like(Z1)
    Z2 = torch.empty(n, dims[2], dtype=tdt, device=dev)
    G2 = torch.empty_like(Z2); G1 = torch.empty_like(H1)
    dW1 = torch.empty(dims[0], dims[1], device=dev); dW2 = torch.empty(dims[1], dims[2], device=dev)
    loss = torch.zeros(1, device=dev)
    say(f"two-layer epoch config 1 bf16={bf16}")
    gcn.gcn_layer_fwd(A, Xd, W1d, H1, act=gcn.ACT_RELU, Z=Z1)
    gcn.gcn_layer_fwd(A, H1, W2d, Z2, act=gcn.ACT_NONE)
    gcn.gcn_softmax_xent(Z2, yd, 1.0 / n, loss, G2)
    gcn.gcn_layer_bwd(A, H1, W2d, G2, dW2, dH=G1, Zprev=Z1)
    gcn.gcn_layer_bwd(A, Xd, W1d, G1, dW1)
    torch.cuda.synchronize()
    f1 = oracle.layer_fwd(og, X, W1, act="relu")
    check_bound(to_np(Z1), f1["Z"], f1["Bz"], tol, "Z1")
    check_bound(to_np(H1), f1["Hout"], f1["Bz"], tol, "H1")
    h1, z1 = to_np(H1), to_np(Z1)
    f2 = oracle.layer_fwd(og, h1, W2, act="none")
    check_bound(to_np(Z2), f2["Z"], f2["Bz"], tol, "Z2")
    z2 = to_np(Z2)
    ol, olabs, oG = oracle.softmax_xent(z2, c1["y"], 1.0 / n)
    assert abs(float(loss.item()) - ol) <= TOL_F32 * max(olabs, np.abs(z2).max() * 3)
    onehot = np.zeros_like(oG); onehot[np.arange(n), c1["y"]] = 1.0 / n
    check_bound(to_np(G2), oG, oG + 2 * onehot, tol, "G2")
    g2 = to_np(G2)
    b2 = oracle.layer_bwd(og, h1, W2, g2, Zprev=z1)
    check_bound(to_np(dW2), b2["dW"], b2["BdW"], tol, "dW2")
    check_bound(to_np(G1), b2["dH"], b2["BdH"], tol, "G1")
    b1 = oracle.layer_bwd(og, X, W1, to_np(G1), want_dH=False)
    check_bound(to_np(dW1), b1["dW"], b1["BdW"], tol, "dW1")
    assert 1.5 < float(loss.item()) < 3.0         # near ln 8 for random weights and labels


# row counts around the kernels' tile and chunk sizes (16-row tiles, 16-row request batches, 512-row splits),
# widths that pick each dense kernel variant (vector requests: d_in a multiple of 4; side-by-side tiles of
# the second operand for d_out up to 64, 128, 256; branch-free product with and without a tail in K and N;
# bf16 features on the bf16 matrix pipe)
@pytest.mark.parametrize("rows", [1, 2, 3, 15, 17, 33, 511, 513, 1025, 8191, 70001])
@pytest.mark.parametrize("d_in,d_out,bf16", [(128, 128, False), (128, 16, False), (16, 128, True), (100, 256, False),
                                               (64, 40, False), (32, 200, True), (36, 129, False), (7, 5, False),
                                               (128, 128, True), (100, 256, True), (256, 47, True), (47, 256, True),
                                               (256, 256, True), (44, 41, True), (47, 256, False), (256, 47, False)])
def test_dense_kernels_over_row_counts(gcn, dev, rows, d_in, d_out, bf16):
    case = Case(gcn, dev, np.zeros(0, np.int32), np.zeros(0, np.int32), rows)          # A^ = I
    run_fwd(gcn, dev, case, d_in, d_out, bf16=bf16, bias=True, save_ah=True)
    run_bwd(gcn, dev, case, d_in, d_out, bf16=bf16, saved_ah=True, dbias=True)
    run_bwd(gcn, dev, case, d_in, d_out, bf16=bf16, want_dh=False)
    case.A.free()
