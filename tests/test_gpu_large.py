"""GPU parity on buffers past 2^32 bytes and past 2^31 elements (the maximum-size edge case).

Every dense buffer of the library is addressed as base + row * leading dimension; a product or an offset
kept in 32 bits would wrap at these sizes and nowhere below.  The buffers here are filled on the GPU (plain
random numbers: no arithmetic of the method), and the oracle recomputes sampled output rows from the
few input rows each of them depends on, copied to the host: rows at the start, around the 2^32-byte mark,
around the 2^31-element mark, at the very end, and random ones.  Sums that run over all rows (the weight
gradient) are made checkable by a gradient that is zero outside those sampled rows, so that the exact
sum has few terms while the kernel still walks every row.

Tolerance as everywhere: |gpu - oracle| <= 1e-5 * (the same sum with absolute values) in fp32, 2e-2 with
bf16 features; copies and graph arrays bit for bit.
"""
import numpy as np
import pytest

import oracle
from util import TOL_BF16, TOL_F32, check_bound, say

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
def release_cached_memory():
    """The buffers here run to tens of GB; hand them back to the driver after each test, since the library
    allocates its own workspaces outside the array library's pool."""
    yield
    import torch
    torch.cuda.empty_cache()


def randn(shape, dev, seed, dtype=None):
    import torch
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    t = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
    return t if dtype is None else t.to(dtype)


def marks(n_rows, row_elems, es):
    """Row numbers around the places where a 32-bit byte or element offset would wrap."""
    out = [0, 1, n_rows - 2, n_rows - 1]
    for k in range(1, 8):
        for at in ((k << 32) // (row_elems * es), (k << 31) // row_elems):
            out += [at - 1, at, at + 1]
    return np.array(sorted({r for r in out if 0 <= r < n_rows}), np.int64)


def sample_rows(n_rows, row_elems, es, n_random, seed):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([marks(n_rows, row_elems, es), rng.integers(0, n_rows, n_random)]))


def rows_to_host(t, rows, dev):
    """Selected rows of a GPU matrix as an fp32 numpy array (bf16 widens exactly)."""
    import torch
    return t[torch.from_numpy(np.ascontiguousarray(rows, np.int64)).to(dev)].float().cpu().numpy()


def compact(ptr, idx, val, rows):
    """The sparse rows `rows` with their column ids renumbered 0..u-1; returns ptr, idx, val, the u old ids."""
    lens = (ptr[rows + 1] - ptr[rows]).astype(np.int64)
    p = np.zeros(rows.size + 1, np.int64)
    p[1:] = np.cumsum(lens)
    sel = np.concatenate([np.arange(ptr[r], ptr[r + 1]) for r in rows]) if rows.size else np.zeros(0, np.int64)
    used, inv = np.unique(idx[sel], return_inverse=True)
    return p, inv.astype(np.int32), val[sel], used.astype(np.int64)


def sparse_rows(ptr, idx, val, rows, X, dev):
    """Oracle product of the sampled sparse rows with the GPU matrix X, and its absolute-value bound."""
    p, j, v, used = compact(ptr, idx, val, rows)
    return oracle.spmm(p, j, v, rows_to_host(X, used, dev))


# ---------------------------------------------------------------------------------------------------------
def test_gather_past_4gib(gcn, dev):
    import torch
    nt, d, n_idx = 17_000_000, 128, 9_000_000        # table 8.7 GB (2.2 G elements), receive buffer 4.6 GB
    say(f"gather table={nt}x{d} fp32 n_idx={n_idx}")
    table = randn((nt, d), dev, 1)
    rng = np.random.default_rng(2)
    idx = rng.integers(0, nt, n_idx).astype(np.int32)
    idx[:4] = [nt - 1, 0, (1 << 32) // (d * 4), (1 << 31) // d]
    idx[-2:] = [nt - 1, (1 << 33) // (d * 4) + 1]
    idx_d = torch.from_numpy(idx).to(dev)
    recv = torch.full((n_idx, d), float("nan"), device=dev)
    gcn.gcn_halo_gather(table, idx_d, recv)
    torch.cuda.synchronize()
    # sampled positions against the oracle's copy
    pos = sample_rows(n_idx, d, 4, 3000, 3)
    src_rows, inv = np.unique(idx[pos], return_inverse=True)
    want = oracle.gather(rows_to_host(table, src_rows, dev), inv.astype(np.int32))
    got = rows_to_host(recv, pos, dev)
    assert np.array_equal(got.view(np.int32), np.asarray(want, np.float32).view(np.int32))
    # every position: the same rows through the array library's own indexing, in slabs
    for s in range(0, n_idx, 1 << 20):
        e = min(n_idx, s + (1 << 20))
        assert torch.equal(recv[s:e].view(torch.int32), table[idx_d[s:e].long()].view(torch.int32)), (s, e)


# ---------------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def wide_block(gcn, dev):
    """A row block whose halo makes the operand of the sparse product 9 GB: 100 k owned rows of a graph on
    40 M vertices, about 30 entries per row, nine in ten of them in columns other blocks own."""
    import torch
    n, lo, nr, per_row = 40_000_000, 20_000_000, 100_000, 30
    rng = np.random.default_rng(5)
    src = np.repeat(np.arange(lo, lo + nr), per_row)
    far = rng.integers(0, n, src.size)
    near = rng.integers(lo, lo + nr, src.size)
    dst = np.where(rng.random(src.size) < 0.9, far, near)
    # degrees of all vertices: the owned ones counted from the edges (distinct neighbours + the self-loop), the
    # others drawn at random (their rows belong to other blocks)
    keep = src != dst
    pairs = np.unique(src[keep].astype(np.int64) * n + dst[keep])
    deg = rng.integers(1, 64, n).astype(np.int32)
    deg[lo:lo + nr] = 1 + np.bincount(pairs // n - lo, minlength=nr)
    say(f"block build n={n} rows=[{lo},{lo + nr}) edges={src.size}")
    og = oracle.graph_build(src, dst, n, lo, lo + nr, deg_global=deg)
    A = gcn.gcn_csr_build(torch.from_numpy(src.astype(np.int32)).to(dev), torch.from_numpy(dst.astype(np.int32)).to(dev),
                          n, lo, lo + nr, deg_global=torch.from_numpy(deg).to(dev))
    return og, A


def test_block_arrays_with_40m_global_ids(wide_block):
    og, A = wide_block
    assert (A.nr, A.nh, A.nnz) == (og.nr, og.nh, og.nnz) and og.nh > 2_000_000
    arr = A.arrays()
    for name in ["rowptr", "col", "deg", "halo_gid", "colptr", "rowidx"]:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name


@pytest.mark.parametrize("bf16", [False, True])
def test_spmm_operand_past_4gib(gcn, dev, wide_block, bf16):
    import torch
    og, A = wide_block
    d = 800 if not bf16 else 1600                      # fp32: 9 GB, 2.2 G elements; bf16: 9 GB, 4.5 G elements
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    assert og.nc * d > (1 << 31)
    say(f"spmm rows={og.nr} cols={og.nc} d={d} bf16={bf16}")
    X = randn((og.nc, d), dev, 7, tdt)
    Y = torch.full((og.nr, d), float("nan"), dtype=tdt, device=dev)
    gcn.gcn_spmm(A, X, Y)
    torch.cuda.synchronize()
    rows = sample_rows(og.nr, d, X.element_size(), 300, 8)
    # the rows whose entries reach the last columns, beyond every 32-bit mark
    last_cols = np.unique(og.rowidx[og.colptr[og.nc - 3]:og.colptr[og.nc]])
    rows = np.unique(np.concatenate([rows, last_cols]))
    ref, bound = sparse_rows(og.rowptr, og.col, og.val, rows, X, dev)
    check_bound(rows_to_host(Y, rows, dev), ref, bound, tol, "A X rows")

    say(f"spmm_t rows={og.nr} cols={og.nc} d={d} bf16={bf16} (output past 4 GiB)")
    G = randn((og.nr, d), dev, 9, tdt)
    D = torch.full((og.nc, d), float("nan"), dtype=tdt, device=dev)
    gcn.gcn_spmm_t(A, G, D)
    torch.cuda.synchronize()
    cols = sample_rows(og.nc, d, X.element_size(), 600, 10)
    ref, bound = sparse_rows(og.colptr, og.rowidx, og.val_t, cols, G, dev)
    check_bound(rows_to_host(D, cols, dev), ref, bound, tol, "A^T G rows")
    assert bool(torch.isfinite(D[-1000:].float()).all()) and bool(torch.isfinite(D[:1000].float()).all())


# ---------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,d_in,d_out,bf16", [
    (17_000_000, 128, 128, False),       # both sides 8.7 GB, 2.2 G elements
    (17_000_000, 16, 128, False),        # short rows in, long rows out
    (17_000_000, 128, 16, False),
    (17_000_000, 128, 128, True),        # bf16: 4.35 GB each
    (9_000_000, 256, 256, False),        # the LDS-tiled kernel: 9.2 GB each
    (11_000_000, 100, 47, False),        # unaligned rows
    (11_000_000, 100, 200, True),
])
def test_dense_fwd_past_4gib(gcn, dev, rows, d_in, d_out, bf16):
    import torch
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    say(f"dense_fwd rows={rows} d_in={d_in} d_out={d_out} bf16={bf16}")
    X = randn((rows, d_in), dev, 11, tdt)
    rng = np.random.default_rng(12)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    Out = torch.full((rows, d_out), float("nan"), dtype=tdt, device=dev)
    Z = torch.full((rows, d_out), float("nan"), dtype=tdt, device=dev)
    gcn.gcn_dense_fwd(X, torch.from_numpy(W).to(dev), Out, bias=torch.from_numpy(b).to(dev), act=gcn.ACT_RELU, Z=Z)
    torch.cuda.synchronize()
    es = X.element_size()
    pick = np.unique(np.concatenate([sample_rows(rows, d_in, es, 2000, 13), marks(rows, d_out, es)]))
    ref, bound = oracle.gemm("nn", rows_to_host(X, pick, dev), W)
    ref = ref + b.astype(np.float64); bound = bound + np.abs(b.astype(np.float64))
    check_bound(rows_to_host(Z, pick, dev), ref, bound, tol, "Z rows")
    check_bound(rows_to_host(Out, pick, dev), np.maximum(ref, 0.0), bound, tol, "Out rows")
    # nothing left unwritten, at either end or in the middle
    for s in (0, rows // 2, rows - 4096):
        assert bool(torch.isfinite(Out[s:s + 4096].float()).all())


# ---------------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def long_graph(gcn, dev):
    """17 M vertices, 3 M undirected edges: most rows hold the self-loop only; what matters is the row count."""
    import torch
    n, m = 17_000_000, 3_000_000
    rng = np.random.default_rng(17)
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    # make sure the rows at the 32-bit marks have neighbours on the far side of them
    near = marks(n, 128, 4)
    u = np.concatenate([u, near]); v = np.concatenate([v, (near + n // 2) % n])
    src = np.concatenate([u, v]).astype(np.int32); dst = np.concatenate([v, u]).astype(np.int32)
    say(f"graph build n={n} directed edges={src.size}")
    og = oracle.graph_build(src, dst, n)
    A = gcn.gcn_csr_build(torch.from_numpy(src).to(dev), torch.from_numpy(dst).to(dev), n)
    assert (A.nr, A.nh, A.nnz) == (og.nr, 0, og.nnz)
    return og, A


@pytest.mark.parametrize("bf16", [False, True])
def test_layer_over_17m_rows(gcn, dev, long_graph, bf16):
    import torch
    og, A = long_graph
    n, d0, d1, d2 = og.nr, 128, 128, 16
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    es = 2 if bf16 else 4
    rng = np.random.default_rng(19)
    W1 = (rng.standard_normal((d0, d1)) / np.sqrt(d0)).astype(np.float32)
    W2 = (rng.standard_normal((d1, d2)) / np.sqrt(d1)).astype(np.float32)
    H0 = randn((n, d0), dev, 20, tdt)

    say(f"layer_fwd rows={n} {d0}->{d1} bf16={bf16}")
    H1 = torch.full((n, d1), float("nan"), dtype=tdt, device=dev)
    AH = torch.full((n, d0), float("nan"), dtype=tdt, device=dev)
    gcn.gcn_layer_fwd(A, H0, torch.from_numpy(W1).to(dev), H1, act=gcn.ACT_RELU, AH_save=AH)
    torch.cuda.synchronize()
    rows = sample_rows(n, d0, es, 1500, 21)
    busy = np.argsort(-np.diff(og.rowptr), kind="stable")[:200]         # the rows with most neighbours
    rows = np.unique(np.concatenate([rows, busy]))
    ax, bax = sparse_rows(og.rowptr, og.col, og.val, rows, H0, dev)
    check_bound(rows_to_host(AH, rows, dev), ax, bax, tol, "saved A^ H rows")
    W1d = W1.astype(np.float64)
    check_bound(rows_to_host(H1, rows, dev), np.maximum(ax @ W1d, 0.0), bax @ np.abs(W1d), tol, "H1 rows")

    # second layer backward over all rows: G is zero outside `win`, so the weight gradient is a sum over those rows
    say(f"layer_bwd rows={n} {d1}->{d2} bf16={bf16}")
    win = np.unique(np.concatenate([m + np.arange(-40, 40) for m in marks(n, d1, es)] + [rng.integers(0, n, 3000)]))
    win = win[(win >= 0) & (win < n)]
    Gw = rng.standard_normal((win.size, d2)).astype(np.float32)
    G = torch.zeros((n, d2), dtype=tdt, device=dev)
    G[torch.from_numpy(win).to(dev)] = torch.from_numpy(Gw).to(dev).to(tdt)
    Gw = rows_to_host(G, win, dev)                                       # as stored (bf16-rounded where it applies)
    dW = torch.full((d1, d2), float("nan"), device=dev)
    D = torch.full((n, d1), float("nan"), dtype=tdt, device=dev)
    gcn.gcn_layer_bwd(A, H1, torch.from_numpy(W2).to(dev), G, dW, dH=D, Zprev=H1)
    torch.cuda.synchronize()
    ah, bah = sparse_rows(og.rowptr, og.col, og.val, win, H1, dev)
    Gd = Gw.astype(np.float64)
    check_bound(dW.cpu().numpy(), ah.T @ Gd, bah.T @ np.abs(Gd), tol, "dW over all rows")
    # dH rows: those that receive something (neighbours of the rows in win) and the sampled ones
    touched = np.unique(og.col[np.concatenate([np.arange(og.rowptr[r], og.rowptr[r + 1]) for r in win])])
    cols = np.unique(np.concatenate([touched[:4000], rows]))
    t, bt = sparse_rows(og.colptr, og.rowidx, og.val_t, cols, G, dev)
    W2d = W2.astype(np.float64)
    S, BS = t @ W2d.T, bt @ np.abs(W2d.T)
    S[~(rows_to_host(H1, cols, dev) > 0)] = 0.0
    check_bound(rows_to_host(D, cols, dev), S, BS, tol, "dH rows")
    assert bool(torch.isfinite(D[-4096:].float()).all())


def test_softmax_past_4gib(gcn, dev):
    import torch
    nr, C = 9_000_000, 128                    # 4.6 GB of logits and as much of gradient
    say(f"softmax_xent rows={nr} C={C}")
    rng = np.random.default_rng(23)
    pick = np.unique(np.concatenate([marks(nr, C, 4), rng.integers(0, nr, 4000)]))
    Z = torch.zeros((nr, C), device=dev)
    Zp = (3.0 * rng.standard_normal((pick.size, C))).astype(np.float32)
    Z[torch.from_numpy(pick).to(dev)] = torch.from_numpy(Zp).to(dev)
    y = rng.integers(0, C, nr).astype(np.int32)
    G = torch.full((nr, C), float("nan"), device=dev)
    loss = torch.zeros(1, device=dev)
    scale = 1.0 / nr
    gcn.gcn_softmax_xent(Z, torch.from_numpy(y).to(dev), scale, loss, G)
    torch.cuda.synchronize()
    lp, labs, Gp = oracle.softmax_xent(Zp, y[pick], scale)
    onehot = np.zeros_like(Gp); onehot[np.arange(pick.size), y[pick]] = scale
    check_bound(rows_to_host(G, pick, dev), Gp, Gp + 2 * onehot, TOL_F32, "G rows")
    # rows of zeros contribute scale * ln C each (closed form), the others what the oracle says
    want = lp + scale * (nr - pick.size) * np.log(C)
    assert abs(float(loss.item()) - want) <= TOL_F32 * (labs + scale * nr * np.log(C)), (float(loss.item()), want)
    rest = torch.ones(nr, dtype=torch.bool, device=dev)
    rest[torch.from_numpy(pick).to(dev)] = False
    # a row of zeros: scale * (1/C - onehot), the same in every such row
    g0 = G[rest]
    yy = torch.from_numpy(y).to(dev)[rest].long()
    base = torch.full((C,), scale / C, device=dev)
    assert torch.allclose(g0.sum(dim=1), torch.zeros(1, device=dev), atol=1e-9)
    assert torch.allclose(g0.gather(1, yy[:, None])[:, 0], (base[0] - scale).expand(g0.shape[0]), rtol=1e-5, atol=0)


# ---------------------------------------------------------------------------------------------------------
# Launches of more than 2^32 threads (2^24 blocks of 256): the runtime would run such a grid modulo 2^32 in one
# dimension, the library folds it into two.  A graph without edges has A^ = I, so both products must return
# their operand bit for bit, and a gather is a copy: closed forms that need no second copy of 35 GB on the host.
def test_products_over_70m_rows_identity(gcn, dev):
    import torch
    n, d = 70_000_000, 128                     # two feature slices: n / 4 = 17.5 M blocks > 2^24
    say(f"identity graph n={n} d={d}")
    empty = torch.zeros(0, dtype=torch.int32, device=dev)
    A = gcn.gcn_csr_build(empty, empty, n)
    assert (A.nr, A.nh, A.nnz) == (n, 0, n)
    arr = A.arrays()
    for name, step in (("rowptr", 1), ("colptr", 1)):
        t = arr[name]
        assert int(t[0]) == 0 and int(t[-1]) == n and bool((t[1:] - t[:-1] == step).all()), name
    for name in ("col", "rowidx"):
        assert bool((arr[name] == torch.arange(n, dtype=torch.int32, device=dev)).all()), name
    assert bool((arr["val"] == 1.0).all()) and bool((arr["deg"] == 1).all())
    X = randn((n, d), dev, 31)
    Y = torch.full((n, d), float("nan"), device=dev)
    gcn.gcn_spmm(A, X, Y)
    torch.cuda.synchronize()
    for s in range(0, n, 1 << 22):
        assert torch.equal(Y[s:s + (1 << 22)].view(torch.int32), X[s:s + (1 << 22)].view(torch.int32)), s
    Y.fill_(float("nan"))
    gcn.gcn_spmm_t(A, X, Y, epilogue=gcn.EPI_RELU)
    torch.cuda.synchronize()
    for s in range(0, n, 1 << 22):
        assert torch.equal(Y[s:s + (1 << 22)], torch.clamp_min(X[s:s + (1 << 22)], 0.0)), s
    A.free()


def test_gather_of_135m_rows(gcn, dev):
    import torch
    nt, d, n_idx = 4096, 128, 135_000_000      # 8 rows per block: 16.9 M blocks > 2^24; 69 GB received
    say(f"gather table={nt}x{d} n_idx={n_idx}")
    table = randn((nt, d), dev, 37)
    gen = torch.Generator(device=dev); gen.manual_seed(38)
    idx = torch.randint(0, nt, (n_idx,), generator=gen, device=dev, dtype=torch.int32)
    recv = torch.full((n_idx, d), float("nan"), device=dev)
    gcn.gcn_halo_gather(table, idx, recv)
    torch.cuda.synchronize()
    for s in range(0, n_idx, 1 << 22):
        e = min(n_idx, s + (1 << 22))
        assert torch.equal(recv[s:e].view(torch.int32), table[idx[s:e].long()].view(torch.int32)), (s, e)
