"""Pins for the CPU oracle: it is checked against what the paper's definitions and plain
mathematics fix (closed forms, dense brute force on tiny graphs, the paper's worked halo
example, finite differences), never against itself or against the GPU path."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def rand_edges(n, m, seed, directed=False):
    rng = np.random.default_rng(seed)
    u = rng.integers(0, n, m)
    v = rng.integers(0, n, m)
    if directed:
        return u.astype(np.int32), v.astype(np.int32)
    return np.concatenate([u, v]).astype(np.int32), np.concatenate([v, u]).astype(np.int32)


def dense_norm_adj(src, dst, n):
    """Sec. 3.1 written out densely in fp64: A^ = D^-1/2 (A + I) D^-1/2, D = row sums of A + I."""
    A = np.zeros((n, n))
    for s, t in zip(src, dst):
        if s != t:
            A[s, t] = 1.0
    At = A + np.eye(n)
    d = At.sum(axis=1)
    return At / np.sqrt(np.outer(d, d)), d, At


def csr_to_dense(g, vals):
    M = np.zeros((g.nr, g.nc))
    for i in range(g.nr):
        for k in range(g.rowptr[i], g.rowptr[i + 1]):
            assert M[i, g.col[k]] == 0.0, "duplicate column in a row"
            M[i, g.col[k]] = vals[k]
    return M


def ulp_diff(a, b):
    a = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    return np.abs(a - b)


# ----------------------------------------------------------------------------- A^ values
@pytest.mark.parametrize("seed,directed", [(1, False), (2, False), (3, True)])
def test_adjacency_matches_dense_definition(seed, directed):
    n = 97
    src, dst = rand_edges(n, 600, seed, directed)
    g = oracle.graph_build(src, dst, n)
    Ad, d, At = dense_norm_adj(src, dst, n)
    # pattern, degrees, fp64 values, fp32 values
    assert np.array_equal(csr_to_dense(g, np.ones(g.nnz)), At)
    assert np.array_equal(g.deg, d.astype(np.int32))
    assert g.nnz == int(At.sum()) == int(g.deg.sum())
    np.testing.assert_allclose(csr_to_dense(g, g.val64), Ad, rtol=1e-15, atol=0)
    assert ulp_diff(csr_to_dense(g, g.val), Ad.astype(np.float32)).max() <= 2
    # columns strictly ascending inside every row
    for i in range(n):
        c = g.col[g.rowptr[i]:g.rowptr[i + 1]]
        assert np.all(np.diff(c) > 0)


def test_closed_forms_ring_complete_star():
    # k-regular ring: every value 1/(k+1), every row sum 1
    n, k = 64, 6
    s = np.repeat(np.arange(n), k)
    t = (s + np.tile(np.concatenate([np.arange(1, k // 2 + 1), -np.arange(1, k // 2 + 1)]), n)) % n
    g = oracle.graph_build(s, t, n)
    assert np.all(g.deg == k + 1)
    np.testing.assert_allclose(g.val64, 1.0 / (k + 1), rtol=1e-15)
    # complete graph: A^ = (1/n) 1 1^T so A^ X = column means
    n = 23
    s, t = np.nonzero(~np.eye(n, dtype=bool))
    g = oracle.graph_build(s, t, n)
    X = np.random.default_rng(0).standard_normal((n, 5)).astype(np.float32)
    Y, _ = oracle.spmm(g.rowptr, g.col, g.val, X)
    np.testing.assert_allclose(Y, np.tile(X.astype(np.float64).mean(0), (n, 1)), rtol=1e-6, atol=1e-7)
    # star: centre degree n (n-1 leaves + itself), leaves degree 2
    n = 50
    leaves = np.arange(1, n)
    s = np.concatenate([np.zeros(n - 1, int), leaves]); t = np.concatenate([leaves, np.zeros(n - 1, int)])
    g = oracle.graph_build(s, t, n)
    assert g.deg[0] == n and np.all(g.deg[1:] == 2)
    row0 = g.val64[g.rowptr[0]:g.rowptr[1]]
    np.testing.assert_allclose(row0[0], 1.0 / n, rtol=1e-15)           # diagonal 1/d_0
    np.testing.assert_allclose(row0[1:], 1.0 / np.sqrt(2.0 * n), rtol=1e-15)


def test_sqrt_degree_is_fixed_vector(c1):
    # sum_j A^(i,j) sqrt(d_j) = sum_{j in N(i)+i} 1/sqrt(d_i) = sqrt(d_i)
    g = oracle.graph_build(c1["src"], c1["dst"], c1["n"])
    sd = np.sqrt(g.deg.astype(np.float64))
    r64 = np.add.reduceat(g.val64 * sd[g.col], g.rowptr[:-1])
    np.testing.assert_allclose(r64, sd, rtol=1e-13)
    Y, _ = oracle.spmm(g.rowptr, g.col, g.val, sd.astype(np.float32)[:, None])
    np.testing.assert_allclose(Y[:, 0], sd, rtol=5e-7)
    # diagonal entries are 1/d_i; symmetric graph => symmetric A^
    diag = np.array([g.val64[g.rowptr[i]:g.rowptr[i + 1]][g.col[g.rowptr[i]:g.rowptr[i + 1]] == i][0]
                     for i in range(0, g.nr, 37)])
    np.testing.assert_allclose(diag, 1.0 / g.deg[::37], rtol=1e-15)


# ----------------------------------------------------------------------------- CSC
def test_csc_of_symmetric_equals_csr_bitwise(c1):
    g = oracle.graph_build(c1["src"], c1["dst"], c1["n"])
    assert np.array_equal(g.colptr, g.rowptr)
    assert np.array_equal(g.rowidx, g.col)
    assert np.array_equal(g.val_t.view(np.int32), g.val.view(np.int32))


def test_csc_of_directed_is_dense_transpose():
    n = 61
    src, dst = rand_edges(n, 400, 7, directed=True)
    g = oracle.graph_build(src, dst, n)
    M = csr_to_dense(g, g.val)
    Mt = np.zeros((n, n), np.float32)
    for j in range(n):
        r = g.rowidx[g.colptr[j]:g.colptr[j + 1]]
        assert np.all(np.diff(r) > 0)
        Mt[j, r] = g.val_t[g.colptr[j]:g.colptr[j + 1]]
    assert np.array_equal(Mt, M.T.astype(np.float32))
    assert not np.array_equal(M, M.T)           # the case really is asymmetric


# ----------------------------------------------------------------------------- halo list
def _read_golden():
    facts = {}
    for line in open(os.path.join(GOLDEN, "halo_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *rest = line.split()
        facts[k] = rest
    return facts


def test_halo_list_paper_worked_example():
    f = _read_golden()
    e = np.array([[int(x) for x in p.split("-")] for p in f["edges"]]) - 1     # 0-based
    src = np.concatenate([e[:, 0], e[:, 1]]); dst = np.concatenate([e[:, 1], e[:, 0]])
    n = 6
    whole = oracle.graph_build(src, dst, n)
    blk = [int(x) - 1 for x in f["block"][0].split(",")]
    g = oracle.graph_build(src, dst, n, blk[0], blk[-1] + 1, deg_global=whole.deg)
    want = [int(x) - 1 for x in f["halo"][0].split(",")]
    assert g.halo_gid.tolist() == want and g.nh == 3
    parts = [[int(x) - 1 for x in p.split(",")] for p in f["parts"]]
    from_p1 = [h for h in g.halo_gid if h in parts[0]]
    from_p2 = [h for h in g.halo_gid if h in parts[1]]
    assert from_p1 == [int(x) - 1 for x in f["halo_from_p1"][0].split(",")]
    assert from_p2 == [int(x) - 1 for x in f["halo_from_p2"][0].split(",")]
    assert len(set(g.halo_gid.tolist())) == g.nh                 # row 4 listed once
    assert whole.deg[0] == int(f["row_weight_v1"][0])
    col2_rows = sorted(whole.rowidx[whole.colptr[1]:whole.colptr[2]] + 1)
    assert col2_rows == [int(x) for x in f["col2_rows"][0].split(",")]
    col4 = sorted(set(whole.rowidx[whole.colptr[3]:whole.colptr[4]] + 1) - {4})
    assert col4 == [int(x) for x in f["col4_offdiag_rows"][0].split(",")]
    # v5 (local row 0) reads owned v5 then halo slots of v1, v4; v6 reads v6 then v2, v4
    assert g.col[g.rowptr[0]:g.rowptr[1]].tolist() == [0, 2 + 0, 2 + 2]
    assert g.col[g.rowptr[1]:g.rowptr[2]].tolist() == [1, 2 + 1, 2 + 2]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_halo_list_brute_force_and_partition_invariance(seed):
    rng = np.random.default_rng(seed)
    n = 120
    src, dst = rand_edges(n, 700, seed, directed=(seed == 13))
    whole = oracle.graph_build(src, dst, n)
    X = rng.standard_normal((n, 7)).astype(np.float32)
    Yw, _ = oracle.spmm(whole.rowptr, whole.col, whole.val, X)
    cuts = [0, 31, 32, 90, n]
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        g = oracle.graph_build(src, dst, n, lo, hi, deg_global=whole.deg)
        cols = set()
        for s, t in zip(src, dst):
            if lo <= s < hi and s != t and not (lo <= t < hi):
                cols.add(int(t))
        assert g.halo_gid.tolist() == sorted(cols)
        assert np.array_equal(g.deg, whole.deg[lo:hi])
        # block form (Sec. 4.1, second equation): owned rows + received rows give the rows of A X
        Xb = np.concatenate([X[lo:hi], X[g.halo_gid]])
        Yb, _ = oracle.spmm(g.rowptr, g.col, g.val, Xb)
        np.testing.assert_allclose(Yb, Yw[lo:hi], rtol=1e-12, atol=1e-13)
        # each row: owned columns first (ascending), then halo slots (ascending)
        for i in range(g.nr):
            assert np.all(np.diff(g.col[g.rowptr[i]:g.rowptr[i + 1]]) > 0)


def test_block_takes_only_halo_degrees_from_the_global_array():
    """D(i,i) is the row sum of A + I (Sec. 3.1) and a row block holds its rows whole (Sec. 4.1): the degrees of
    owned vertices are counted, the global array only serves the halo vertices.  A block built with placeholders in
    the owned positions must equal the block built with the whole graph's degrees, value for value, and both must
    equal the rows of the dense definition."""
    n, lo, hi = 40, 12, 29
    src, dst = rand_edges(n, 150, 5)
    whole = oracle.graph_build(src, dst, n)
    Ad, _, _ = dense_norm_adj(src, dst, n)
    marked = whole.deg.copy(); marked[lo:hi] = 1
    a = oracle.graph_build(src, dst, n, lo, hi, deg_global=whole.deg)
    b = oracle.graph_build(src, dst, n, lo, hi, deg_global=marked)
    assert np.array_equal(a.val.view(np.int32), b.val.view(np.int32)) and np.array_equal(a.val64, b.val64)
    assert np.array_equal(b.deg, whole.deg[lo:hi])
    gid = np.concatenate([np.arange(lo, hi), b.halo_gid])
    for i in range(b.nr):
        for k in range(b.rowptr[i], b.rowptr[i + 1]):
            assert abs(b.val64[k] - Ad[lo + i, gid[b.col[k]]]) <= 1e-15
    # a wrong halo degree, on the other hand, must show
    wrong = marked.copy(); wrong[b.halo_gid[0]] += 3
    c = oracle.graph_build(src, dst, n, lo, hi, deg_global=wrong)
    assert not np.array_equal(c.val64, b.val64)


def test_graph_build_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.graph_build([0, 5], [1, 2], 4)
    with pytest.raises(ValueError):
        oracle.graph_build([0, 1], [1, 0], 4, 0, 2)          # block without global degrees


def test_duplicates_and_self_loops_collapse():
    src = [0, 0, 0, 1, 2, 2, 2]; dst = [1, 1, 0, 0, 2, 0, 0]
    g = oracle.graph_build(src, dst, 3)
    assert g.rowptr.tolist() == [0, 2, 4, 6]
    assert g.col.tolist() == [0, 1, 0, 1, 0, 2]
    assert g.deg.tolist() == [2, 2, 2]


# ----------------------------------------------------------------------------- SpMM
def test_spmm_against_dense_and_adjoint():
    n = 83
    src, dst = rand_edges(n, 500, 21, directed=True)
    g = oracle.graph_build(src, dst, n)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((n, 9)).astype(np.float32)
    Yv = rng.standard_normal((n, 9)).astype(np.float32)
    M = csr_to_dense(g, g.val.astype(np.float64))
    Y, B = oracle.spmm(g.rowptr, g.col, g.val, X)
    np.testing.assert_allclose(Y, M @ X.astype(np.float64), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(B, np.abs(M) @ np.abs(X.astype(np.float64)), rtol=1e-13)
    Yt, _ = oracle.spmm(g.colptr, g.rowidx, g.val_t, Yv)
    np.testing.assert_allclose(Yt, M.T @ Yv.astype(np.float64), rtol=1e-13, atol=1e-14)
    # <Yv, A X> = <A^T Yv, X>
    np.testing.assert_allclose((Yv.astype(np.float64) * Y).sum(), (Yt * X.astype(np.float64)).sum(), rtol=1e-11)
    # row subset
    rows = np.array([5, 0, 82, 5])
    Ys, _ = oracle.spmm(g.rowptr, g.col, g.val, X, rows=rows)
    np.testing.assert_array_equal(Ys, Y[rows])


# ----------------------------------------------------------------------------- dense products
def test_gemm_forms():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((13, 7)).astype(np.float32)
    B = rng.standard_normal((7, 5)).astype(np.float32)
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    C, Bd = oracle.gemm("nn", A, B)
    np.testing.assert_allclose(C, A64 @ B64, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(Bd, np.abs(A64) @ np.abs(B64), rtol=1e-13)
    C, _ = oracle.gemm("nt", A, B.T.copy())
    np.testing.assert_allclose(C, A64 @ B64, rtol=1e-13, atol=1e-14)
    C, _ = oracle.gemm("tn", A.T.copy(), B)
    np.testing.assert_allclose(C, A64 @ B64, rtol=1e-13, atol=1e-14)
    # identity and one-hot weights
    C, _ = oracle.gemm("nn", A, np.eye(7, dtype=np.float32))
    np.testing.assert_array_equal(C, A64)
    sel = np.zeros((7, 2), np.float32); sel[3, 0] = 1; sel[6, 1] = 1
    C, _ = oracle.gemm("nn", A, sel)
    np.testing.assert_array_equal(C, A64[:, [3, 6]])
    # a non-square transposed case cannot be confused with the plain one
    C, _ = oracle.gemm("tn", A, rng.standard_normal((13, 4)).astype(np.float32))
    assert C.shape == (7, 4)
    # the fp64-operand forms (used where a factor is itself an fp64 result): same three products, and one-hot
    # selectors pick out columns / rows exactly, so a transposed operand or a swapped index cannot pass
    A64b = rng.standard_normal((13, 7)); B64b = rng.standard_normal((7, 5))
    np.testing.assert_allclose(oracle.gemm_dd("nn", A64b, B64b), A64b @ B64b, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.gemm_dd("nt", A64b, B64b.T.copy()), A64b @ B64b, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.gemm_dd("tn", A64b.T.copy(), B64b), A64b @ B64b, rtol=1e-13, atol=1e-14)
    np.testing.assert_array_equal(oracle.gemm_dd("nn", A64b, sel.astype(np.float64)), A64b[:, [3, 6]])
    np.testing.assert_array_equal(oracle.gemm_dd("nt", A64b, sel.T.astype(np.float64).copy()), A64b[:, [3, 6]])
    rsel = np.zeros((13, 2)); rsel[2, 0] = 1; rsel[11, 1] = 1
    np.testing.assert_array_equal(oracle.gemm_dd("tn", rsel, A64b), A64b[[2, 11], :])


# ----------------------------------------------------------------------------- softmax cross-entropy
def test_softmax_xent_closed_forms():
    nr, C = 37, 8
    y = (np.arange(nr) % C).astype(np.int32)
    scale = 1.0 / nr
    loss, labs, G = oracle.softmax_xent(np.zeros((nr, C), np.float32), y, scale)
    np.testing.assert_allclose(loss, np.log(C), rtol=1e-14)
    np.testing.assert_allclose(labs, np.log(C), rtol=1e-14)
    want = np.full((nr, C), scale / C); want[np.arange(nr), y] -= scale
    np.testing.assert_allclose(G, want, rtol=1e-14)
    rng = np.random.default_rng(9)
    Z = (3 * rng.standard_normal((nr, C))).astype(np.float32)
    l1, _, G1 = oracle.softmax_xent(Z, y, scale)
    np.testing.assert_allclose(G1.sum(1), 0.0, atol=1e-16)
    l2, _, G2 = oracle.softmax_xent(Z + np.float32(4.0), y, scale)      # shift invariance
    np.testing.assert_allclose(l2, l1, rtol=1e-6); np.testing.assert_allclose(G2, G1, atol=1e-7)
    # unlabeled rows
    y2 = y.copy(); y2[::3] = -1
    l3, _, G3 = oracle.softmax_xent(Z, y2, scale)
    assert np.all(G3[::3] == 0) and np.array_equal(G3[1::3], G1[1::3]) and l3 < l1
    # direct formula in numpy fp64
    Zd = Z.astype(np.float64)
    lse = np.log(np.exp(Zd).sum(1))
    np.testing.assert_allclose(l1, scale * (lse - Zd[np.arange(nr), y]).sum(), rtol=1e-13)


def test_softmax_xent_finite_differences():
    nr, C = 9, 5
    rng = np.random.default_rng(4)
    Z = rng.standard_normal((nr, C)).astype(np.float32)
    y = rng.integers(0, C, nr).astype(np.int32)
    _, _, G = oracle.softmax_xent(Z, y, 0.7)

    def J(Zd):
        return 0.7 * (np.log(np.exp(Zd).sum(1)) - Zd[np.arange(nr), y]).sum()
    Zd = Z.astype(np.float64); h = 1e-6
    for i in range(nr):
        for c in range(C):
            E = np.zeros_like(Zd); E[i, c] = h
            fd = (J(Zd + E) - J(Zd - E)) / (2 * h)
            assert abs(fd - G[i, c]) <= 1e-8 + 1e-6 * abs(fd)


# ----------------------------------------------------------------------------- layer forward / backward
def _dense_two_layer(Ad, X, W1, W2, y, scale):
    """Independent fp64 forward pass written with dense numpy (Sec. 3.1, first equation, twice)."""
    Z1 = Ad @ X @ W1
    H1 = np.maximum(Z1, 0.0)
    Z2 = Ad @ H1 @ W2
    lse = np.log(np.exp(Z2 - Z2.max(1, keepdims=True)).sum(1)) + Z2.max(1)
    return scale * (lse - Z2[np.arange(len(y)), y]).sum(), Z1, H1, Z2


@pytest.mark.parametrize("directed", [False, True])
def test_layer_formulas_by_finite_differences(directed):
    n, d0, d1, d2 = 40, 6, 5, 4
    src, dst = rand_edges(n, 160, 31, directed)
    g = oracle.graph_build(src, dst, n)
    Ad = csr_to_dense(g, g.val.astype(np.float64))
    rng = np.random.default_rng(8)
    X = rng.standard_normal((n, d0)).astype(np.float32)
    W1 = (0.5 * rng.standard_normal((d0, d1))).astype(np.float32)
    W2 = (0.5 * rng.standard_normal((d1, d2))).astype(np.float32)
    y = rng.integers(0, d2, n).astype(np.int32)
    scale = 1.0 / n
    J0, Z1d, H1d, Z2d = _dense_two_layer(Ad, X.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64), y, scale)

    # oracle forward (fp64 outputs), layer by layer on the exact fp64 chain where possible
    f1 = oracle.layer_fwd(g, X, W1, act="relu")
    np.testing.assert_allclose(f1["Z"], Z1d, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f1["Hout"], H1d, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f1["AH"], Ad @ X.astype(np.float64), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f1["Bz"], np.abs(Ad) @ np.abs(X.astype(np.float64)) @ np.abs(W1.astype(np.float64)), rtol=1e-12)
    # the other association gives the same numbers
    P, _ = oracle.gemm("nn", X, W1)
    np.testing.assert_allclose(Ad @ P, f1["Z"], rtol=1e-12, atol=1e-13)

    # To finite-difference the whole chain the fp32 hand-over between layers must not round:
    # use fp32-representable H1 by recomputing the dense chain from the rounded values.
    H1 = f1["Hout"].astype(np.float32)
    Z1 = f1["Z"].astype(np.float32)
    f2 = oracle.layer_fwd(g, H1, W2, act="none")
    loss, _, G2 = oracle.softmax_xent(f2["Z"].astype(np.float32), y, scale)
    b2 = oracle.layer_bwd(g, H1, W2, G2.astype(np.float32), Zprev=Z1, want_dH=True, want_dbias=True)
    G1 = b2["dH"].astype(np.float32)
    b1 = oracle.layer_bwd(g, X, W1, G1, Zprev=None, want_dH=True)

    # central differences on the dense fp64 model, entries near a ReLU kink excluded
    h = 1e-6
    X64, W164, W264 = X.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64)

    def Jof(Xp=X64, W1p=W164, W2p=W264):
        return _dense_two_layer(Ad, Xp, W1p, W2p, y, scale)[0]
    assert np.abs(Z1d).min() > 1e-4
    tol = lambda fd: 2e-6 * abs(fd) + 2e-8     # fp32 hand-overs between the layer calls
    for k in range(d1):
        for c in range(d2):
            E = np.zeros_like(W264); E[k, c] = h
            fd = (Jof(W2p=W264 + E) - Jof(W2p=W264 - E)) / (2 * h)
            assert abs(fd - b2["dW"][k, c]) <= tol(fd), ("dW2", k, c, fd, b2["dW"][k, c])
    for k in range(d0):
        for c in range(d1):
            E = np.zeros_like(W164); E[k, c] = h
            fd = (Jof(W1p=W164 + E) - Jof(W1p=W164 - E)) / (2 * h)
            assert abs(fd - b1["dW"][k, c]) <= tol(fd), ("dW1", k, c, fd, b1["dW"][k, c])
    for j in range(0, n, 3):
        for k in range(d0):
            E = np.zeros_like(X64); E[j, k] = h
            fd = (Jof(Xp=X64 + E) - Jof(Xp=X64 - E)) / (2 * h)
            assert abs(fd - b1["dH"][j, k]) <= tol(fd), ("dX", j, k, fd, b1["dH"][j, k])
    # dbias = column sums of G
    np.testing.assert_allclose(b2["dbias"], G2.astype(np.float32).astype(np.float64).sum(0), rtol=1e-12, atol=1e-15)
    # mask really applied: dH of layer 2 is zero exactly where Z1 <= 0
    assert np.all(b2["dH"][Z1 <= 0] == 0.0) and np.any(Z1 <= 0) and np.any(b2["dH"] != 0)


def test_layer_backward_on_blocks_sums_to_whole():
    """Sec. 4.2: the per-processor dW_m add up to dW; dH rows (owned + pushed halo parts) add up to S."""
    n, d_in, d_out = 90, 5, 3
    src, dst = rand_edges(n, 420, 41, directed=True)
    whole = oracle.graph_build(src, dst, n)
    rng = np.random.default_rng(2)
    H = rng.standard_normal((n, d_in)).astype(np.float32)
    W = rng.standard_normal((d_in, d_out)).astype(np.float32)
    G = rng.standard_normal((n, d_out)).astype(np.float32)
    bw = oracle.layer_bwd(whole, H, W, G, Zprev=None)
    dW = np.zeros((d_in, d_out)); S = np.zeros((n, d_in))
    Zw = oracle.layer_fwd(whole, H, W, act="none")["Z"]
    for lo, hi in [(0, 30), (30, 31), (31, 90)]:
        g = oracle.graph_build(src, dst, n, lo, hi, deg_global=whole.deg)
        Hb = np.concatenate([H[lo:hi], H[g.halo_gid]])
        b = oracle.layer_bwd(g, Hb, W, G[lo:hi], Zprev=None)
        dW += b["dW"]
        S[lo:hi] += b["dH"][: g.nr]
        S[g.halo_gid] += b["dH"][g.nr:]
        np.testing.assert_allclose(oracle.layer_fwd(g, Hb, W, act="none")["Z"], Zw[lo:hi], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, bw["dW"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(S, bw["dH"], rtol=1e-11, atol=1e-12)


def test_pull_backward_equals_gradient_on_symmetric_graph_and_adds_up_over_blocks():
    """Algorithm 2 (pull form) on a symmetric A^: on the whole graph it must equal the push form, which the
    finite differences above pin; on row blocks the dH rows are the whole graph's rows (complete, unlike the
    push form) and the dW_m add up to dW."""
    n, d_in, d_out = 80, 6, 4
    src, dst = rand_edges(n, 300, 43)                    # undirected
    whole = oracle.graph_build(src, dst, n)
    assert np.array_equal(whole.rowptr, whole.colptr) and np.array_equal(whole.col, whole.rowidx)
    rng = np.random.default_rng(5)
    H = rng.standard_normal((n, d_in)).astype(np.float32)
    W = rng.standard_normal((d_in, d_out)).astype(np.float32)
    G = rng.standard_normal((n, d_out)).astype(np.float32)
    Zp = rng.standard_normal((n, d_in)).astype(np.float32)
    push = oracle.layer_bwd(whole, H, W, G, Zprev=Zp)
    pull = oracle.layer_bwd_pull(whole, H, W, G, Zprev=Zp)
    np.testing.assert_allclose(pull["dH"], push["dH"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(pull["dW"], push["dW"], rtol=1e-11, atol=1e-12)
    assert np.all(pull["dH"][Zp <= 0] == 0.0) and np.any(pull["dH"] != 0)
    assert np.all(pull["BdH"] >= np.abs(pull["dH"])) and np.all(pull["BdW"] >= np.abs(pull["dW"]) - 1e-12)
    dW = np.zeros((d_in, d_out))
    for lo, hi in [(0, 25), (25, 26), (26, 80)]:
        g = oracle.graph_build(src, dst, n, lo, hi, deg_global=whole.deg)
        b = oracle.layer_bwd_pull(g, H[lo:hi], W, np.concatenate([G[lo:hi], G[g.halo_gid]]), Zprev=Zp[lo:hi])
        np.testing.assert_allclose(b["dH"], push["dH"][lo:hi], rtol=1e-11, atol=1e-12)
        dW += b["dW"]
    np.testing.assert_allclose(dW, push["dW"], rtol=1e-11, atol=1e-12)
    # on a directed graph the pull form is a different quantity (it multiplies by A^, the gradient by A^^T)
    src, dst = rand_edges(n, 300, 44, directed=True)
    gd = oracle.graph_build(src, dst, n)
    assert np.abs(oracle.layer_bwd_pull(gd, H, W, G)["dH"] - oracle.layer_bwd(gd, H, W, G)["dH"]).max() > 1e-3


def test_bias_and_identity_activation():
    n = 30
    src, dst = rand_edges(n, 100, 51)
    g = oracle.graph_build(src, dst, n)
    rng = np.random.default_rng(1)
    H = rng.standard_normal((n, 4)).astype(np.float32)
    W = rng.standard_normal((4, 3)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    f0 = oracle.layer_fwd(g, H, W, act="none")
    f1 = oracle.layer_fwd(g, H, W, bias=b, act="none")
    np.testing.assert_allclose(f1["Z"] - f0["Z"], np.tile(b.astype(np.float64), (n, 1)), atol=1e-14)
    assert np.array_equal(f0["Z"], f0["Hout"])
    fr = oracle.layer_fwd(g, H, W, act="relu")
    assert np.array_equal(fr["Hout"], np.maximum(fr["Z"], 0.0)) and np.any(fr["Z"] < 0)


# ----------------------------------------------------------------------------- gather
def test_gather_identity_and_round_trip():
    rng = np.random.default_rng(6)
    T = rng.standard_normal((50, 6)).astype(np.float32)
    assert np.array_equal(oracle.gather(T, np.arange(50)), T)
    p = rng.permutation(50); inv = np.argsort(p)
    assert np.array_equal(oracle.gather(oracle.gather(T, p), inv), T)
    assert np.array_equal(oracle.gather(T, [3, 3, 49]), T[[3, 3, 49]])
    with pytest.raises(ValueError):
        oracle.gather(T, [50])


# ---- weight update and training loop (Sec. 3.1 last equation; Algorithm 2's update line) ----------------
def test_sgd_update_closed_form():
    W = np.array([[1.0, -2.0], [0.5, 4.0]], np.float32); dW = np.array([[2.0, 2.0], [-1.0, 8.0]], np.float32)
    assert np.array_equal(oracle.sgd_update(W, dW, 0.25), np.array([[0.5, -2.5], [0.75, 2.0]], np.float32))


def test_one_layer_on_an_edgeless_graph_is_softmax_regression():
    """No edges: A + I = I and every degree is 1, so A^ = I and a one-layer GCN is multinomial logistic
    regression; one training step must equal the textbook update W - lr X^T (softmax(XW) - Y) / n."""
    rng = np.random.default_rng(4)
    n, d, c = 50, 6, 4
    e = np.zeros(0, np.int32)
    g = oracle.graph_build(e, e, n)
    assert np.array_equal(g.col, np.arange(n)) and np.all(g.val == 1.0)
    X = rng.standard_normal((n, d)).astype(np.float32); W = rng.standard_normal((d, c)).astype(np.float32)
    y = rng.integers(0, c, n).astype(np.int32)
    losses, (W1,) = oracle.train(g, X, [W], y, lr=0.3, epochs=1)
    Z = X.astype(np.float64) @ W.astype(np.float64)
    Z = Z.astype(np.float32).astype(np.float64)              # the stored pre-activation is fp32
    P = np.exp(Z - Z.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    Y = np.eye(c)[y]
    want_loss = -np.mean(np.log(P[np.arange(n), y]))
    G = ((P - Y) / n).astype(np.float32).astype(np.float64)  # the stored gradient is fp32
    want_W = (W.astype(np.float64) - 0.3 * (X.astype(np.float64).T @ G)).astype(np.float32)
    assert abs(losses[0] - want_loss) <= 1e-12 * abs(want_loss)
    assert np.array_equal(W1, want_W)


def _dense_loss(Ad, X, Ws, y, scale):
    """Independent fp64 model with any number of layers, dense numpy only (Sec. 3.1: H^k = relu(A^ H^(k-1) W^k) for
    k < L, identity on layer L, softmax cross-entropy on Z^L)."""
    H = X
    for k, W in enumerate(Ws):
        Z = Ad @ H @ W
        H = Z if k == len(Ws) - 1 else np.maximum(Z, 0.0)
    lse = np.log(np.exp(Z - Z.max(1, keepdims=True)).sum(1)) + Z.max(1)
    return scale * (lse - Z[np.arange(len(y)), y]).sum()


@pytest.mark.parametrize("dims,directed", [((6, 5, 4), False), ((6, 5, 4), True), ((5, 6, 4, 3), False)])
def test_training_step_with_several_layers_is_gradient_descent_on_the_dense_model(dims, directed):
    """oracle.train itself, for L = 2 and L = 3 (Sec. 3.1 last equation, W <- W - lr dJ/dW; Algorithm 2's update
    line): after one epoch every weight must equal W - lr * (central difference of the dense fp64 loss), and the
    loss it reports must be the dense model's.  A second epoch must be the same step taken from the new weights.
    A dropped ReLU mask, a wrong gradient hand-over between layers or a transposed product changes dJ/dW."""
    n, lr = 36, 0.4
    src, dst = rand_edges(n, 150, 77, directed)
    g = oracle.graph_build(src, dst, n)
    Ad = csr_to_dense(g, g.val.astype(np.float64))
    rng = np.random.default_rng(21)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    Ws = [(0.6 * rng.standard_normal((dims[k], dims[k + 1]))).astype(np.float32) for k in range(len(dims) - 1)]
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    scale = 1.0 / n
    X64 = X.astype(np.float64)

    def check_step(W_before, W_after, loss_reported):
        W64 = [W.astype(np.float64) for W in W_before]
        J0 = _dense_loss(Ad, X64, W64, y, scale)
        assert abs(loss_reported - J0) <= 1e-6 * abs(J0)            # stored layer outputs are fp32
        # no pre-activation may sit on a ReLU kink, or the central difference is not the derivative
        H = X64
        for W in W64[:-1]:
            Z = Ad @ H @ W
            assert np.abs(Z).min() > 1e-4
            H = np.maximum(Z, 0.0)
        h = 1e-6
        for k, W in enumerate(W64):
            for i in range(W.shape[0]):
                for c in range(W.shape[1]):
                    E = np.zeros_like(W); E[i, c] = h
                    Wp = list(W64); Wm = list(W64)
                    Wp[k] = W + E; Wm[k] = W - E
                    fd = (_dense_loss(Ad, X64, Wp, y, scale) - _dense_loss(Ad, X64, Wm, y, scale)) / (2 * h)
                    step = (float(W_before[k][i, c]) - float(W_after[k][i, c])) / lr
                    # fp32 hand-overs between the layer calls, the fp32 rounding of the new weight, the difference quotient
                    tol = 4e-6 * abs(fd) + 4e-8 + 1.2e-7 * abs(float(W_before[k][i, c])) / lr
                    assert abs(step - fd) <= tol, (k, i, c, step, fd)

    losses1, W1 = oracle.train(g, X, Ws, y, lr=lr, epochs=1)
    assert any(np.any(a != b) for a, b in zip(Ws, W1))
    check_step(Ws, W1, losses1[0])
    losses2, W2 = oracle.train(g, X, Ws, y, lr=lr, epochs=2)
    assert losses2[0] == losses1[0]
    check_step(W1, W2, losses2[1])
    # and it is bit for bit one more epoch from where the first stopped
    _, W2b = oracle.train(g, X, W1, y, lr=lr, epochs=1)
    assert all(np.array_equal(a, b) for a, b in zip(W2, W2b))


def test_training_loss_falls_on_a_small_graph():
    rng = np.random.default_rng(8)
    n = 200
    u = rng.integers(0, n, 800); v = rng.integers(0, n, 800)
    g = oracle.graph_build(np.concatenate([u, v]), np.concatenate([v, u]), n)
    X = rng.standard_normal((n, 12)).astype(np.float32)
    Ws = [(rng.standard_normal((12, 8)) * 0.4).astype(np.float32), (rng.standard_normal((8, 3)) * 0.4).astype(np.float32)]
    y = rng.integers(0, 3, n).astype(np.int32)
    losses, _ = oracle.train(g, X, Ws, y, lr=0.5, epochs=25)
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
    assert losses[-1] < losses[0] - 0.01          # labels are random: little can be learnt, but the loss must move


# ----------------------------------------------------------------------------- partition statistics
def _brute_stats(M, part, p):
    """Dense 0/1 matrix, straight from the definitions: who needs row j, who owns it."""
    n = M.shape[0]
    need = np.zeros((p, n), bool)                         # need[q, j]: part q has a row with an entry in column j
    for i in range(n):
        for j in range(n):
            if M[i, j]:
                need[part[i], j] = True
    send = np.zeros(p, int); recv = np.zeros(p, int); talk = np.zeros((p, p), bool)
    for j in range(n):
        for q in range(p):
            if need[q, j] and q != part[j]:
                send[part[j]] += 1; recv[q] += 1; talk[part[j], q] = True
    return send, recv, talk.sum(1), talk.sum(0)


def test_partition_stats_paper_example_and_brute_force():
    f = _read_golden()
    e = np.array([[int(x) for x in q.split("-")] for q in f["edges"]]) - 1
    src = np.concatenate([e[:, 0], e[:, 1]]); dst = np.concatenate([e[:, 1], e[:, 0]])
    g = oracle.graph_build(src, dst, 6)
    part = np.zeros(6, int)
    for m, q in enumerate(f["parts"]):
        part[[int(x) - 1 for x in q.split(",")]] = m
    st = oracle.partition_stats(g.colptr, g.rowidx, g.rowptr, part, 3)
    # printed: lambda(n_2) = lambda(n_4) = 3, row 4 is transferred twice; processor 3 receives rows {1, 2} and {4}
    lam = [len(set(part[g.rowidx[g.colptr[j]:g.colptr[j + 1]]].tolist())) for j in range(6)]
    assert lam[1] == int(f["lambda_n2"][0]) and lam[3] == int(f["lambda_n4"][0])
    assert st["volume"] == sum(lam) - 6
    assert st["recv_rows"][2] == 3 and st["recv_msgs"][2] == 2
    # part 2 owns v3 and v4; v3 has no neighbour outside its part, so all that part 2 sends is row 4, twice
    assert st["send_rows"][1] == int(f["transfers_row4"][0]) and st["send_msgs"][1] == 2
    cut_at_v4 = sum(1 for a, b in e if 3 in (a, b) and part[a] != part[b])
    assert cut_at_v4 == int(f["cut_edges_at_v4"][0]) and lam[3] - 1 == int(f["transfers_row4"][0])
    assert st["volume"] <= st["cut_entries"]                  # the graph model never undercounts
    assert st["load"].tolist() == [int(g.deg[part == m].sum()) for m in range(3)]
    # brute force from a dense matrix, directed graphs, uneven parts, an empty part
    for seed, n, m, p in [(1, 17, 40, 4), (2, 30, 120, 5), (3, 9, 30, 9), (4, 25, 60, 1)]:
        src, dst = rand_edges(n, m, seed, directed=True)
        g = oracle.graph_build(src, dst, n)
        rng = np.random.default_rng(seed)
        part = rng.integers(0, max(p - 1, 1), n) if p > 2 else rng.integers(0, p, n)     # last part stays empty
        M = csr_to_dense(g, g.val) != 0
        st = oracle.partition_stats(g.colptr, g.rowidx, g.rowptr, part, p)
        send, recv, smsg, rmsg = _brute_stats(M, part, p)
        assert st["send_rows"].tolist() == send.tolist() and st["recv_rows"].tolist() == recv.tolist()
        assert st["send_msgs"].tolist() == smsg.tolist() and st["recv_msgs"].tolist() == rmsg.tolist()
        assert st["volume"] == send.sum() and st["cut_entries"] == sum(M[i, j] and part[i] != part[j] for i in range(n) for j in range(n))
        assert st["load"].sum() == g.nnz
    # one part: nothing moves; every vertex its own part: net j reaches deg_j parts
    g = oracle.graph_build(*rand_edges(40, 150, 9), 40)
    st = oracle.partition_stats(g.colptr, g.rowidx, g.rowptr, np.zeros(40, int), 1)
    assert st["volume"] == 0 and st["send_msgs"].sum() == 0 and st["load"][0] == g.nnz
    st = oracle.partition_stats(g.colptr, g.rowidx, g.rowptr, np.arange(40), 40)
    assert st["volume"] == g.nnz - 40 and st["send_rows"].tolist() == (g.deg - 1).tolist()


def test_partition_stats_agree_with_block_halo_lists():
    """Contiguous parts: the rows a part receives are the halo list of its block build (pinned above)."""
    n = 300
    src, dst = rand_edges(n, 1500, 12, directed=True)
    whole = oracle.graph_build(src, dst, n)
    cuts = [0, 70, 71, 190, 300]
    part = np.zeros(n, int)
    for m in range(4):
        part[cuts[m]:cuts[m + 1]] = m
    st = oracle.partition_stats(whole.colptr, whole.rowidx, whole.rowptr, part, 4)
    for m in range(4):
        g = oracle.graph_build(src, dst, n, cuts[m], cuts[m + 1], deg_global=whole.deg)
        assert st["recv_rows"][m] == g.nh and st["load"][m] == g.nnz
        assert st["recv_msgs"][m] == len(set(part[g.halo_gid].tolist()))


# ----------------------------------------------------------------------------- induced subgraphs
def test_induced_subgraph_is_the_dense_submatrix():
    """Sec. 4.3.3: the mini-batch graph has the edges between selected vertices; checked entry by entry against
    the dense pattern restricted to the selection, with the normalisation recomputed from its own row sums."""
    for seed, n, m, k, directed in [(1, 40, 200, 13, True), (2, 60, 500, 60, False), (3, 25, 90, 1, True), (4, 30, 0, 7, False)]:
        src, dst = rand_edges(n, m, seed, directed=directed) if m else (np.zeros(0, np.int32), np.zeros(0, np.int32))
        P = np.zeros((n, n), bool)
        P[src, dst] = True
        np.fill_diagonal(P, False)
        rng = np.random.default_rng(seed)
        V = rng.permutation(n)[:k]
        s2, d2 = oracle.induced_edges(src, dst, n, V)
        g = oracle.graph_build(s2, d2, k)
        sub = P[np.ix_(V, V)] | np.eye(k, dtype=bool)
        deg = sub.sum(1)
        want = np.where(sub, 1.0 / np.sqrt(np.outer(deg, deg)), 0.0)
        got = csr_to_dense(g, g.val64)
        assert np.array_equal(got != 0, sub) and np.array_equal(g.deg, deg)
        np.testing.assert_allclose(got, want, rtol=1e-14)
    # every vertex in its own order: the graph itself; a permutation: the symmetric permutation of A^
    src, dst = rand_edges(35, 150, 8, directed=True)
    whole = oracle.graph_build(src, dst, 35)
    same = oracle.graph_build(*oracle.induced_edges(src, dst, 35, np.arange(35)), 35)
    assert np.array_equal(same.col, whole.col) and np.array_equal(same.val, whole.val)
    perm = np.random.default_rng(0).permutation(35)
    gp = oracle.graph_build(*oracle.induced_edges(src, dst, 35, perm), 35)
    assert np.array_equal(csr_to_dense(gp, gp.val), csr_to_dense(whole, whole.val)[np.ix_(perm, perm)])


# ----------------------------------------------------------------------------- the tolerance bounds themselves
@pytest.mark.parametrize("directed", [False, True])
def test_bounds_are_the_sums_of_absolute_terms(directed):
    """Every parity test allows tol * B, so a B that is too large would hollow out all of them: each bound the
    oracle returns is the same sum with every factor replaced by its absolute value, written out densely here."""
    n, lo, hi, d_in, d_out = 60, 10, 45, 7, 5
    src, dst = rand_edges(n, 260, 41, directed)
    whole = oracle.graph_build(src, dst, n)
    g = oracle.graph_build(src, dst, n, lo, hi, deg_global=whole.deg)
    assert g.nh > 0
    M = np.abs(csr_to_dense(g, g.val.astype(np.float64)))            # |A^_m|, nr x nc
    rng = np.random.default_rng(11)
    H = rng.standard_normal((g.nc, d_in)).astype(np.float32)
    W = rng.standard_normal((d_in, d_out)).astype(np.float32)
    G = rng.standard_normal((g.nr, d_out)).astype(np.float32)
    Zp = rng.standard_normal((g.nr, d_in)).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    aH, aW, aG = (np.abs(x.astype(np.float64)) for x in (H, W, G))

    f = oracle.layer_fwd(g, H, W, bias=b, act="relu")
    np.testing.assert_allclose(f["Bz"], M @ aH @ aW + np.abs(b.astype(np.float64)), rtol=1e-12)

    bw = oracle.layer_bwd(g, H, W, G, Zprev=Zp, want_dH=True, want_dbias=True)
    np.testing.assert_allclose(bw["BdW"], (M @ aH).T @ aG, rtol=1e-12)
    np.testing.assert_allclose(bw["Bdb"], aG.sum(0), rtol=1e-12)
    BdH = M.T @ aG @ aW.T                                           # all nc rows, mask or no mask
    keep = np.ones((g.nc, d_in), bool); keep[: g.nr] = Zp > 0
    np.testing.assert_allclose(bw["BdH"][keep], BdH[keep], rtol=1e-12)
    assert np.all(bw["BdH"] <= BdH * (1 + 1e-12))                   # a masked element may carry its bound or none
    assert np.all(np.abs(bw["dW"]) <= bw["BdW"]) and np.all(np.abs(bw["dH"]) <= bw["BdH"] + 1e-300)

    A = rng.standard_normal((13, 7)).astype(np.float32); B = rng.standard_normal((7, 5)).astype(np.float32)
    aA, aB = np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64))
    for op, x, y in (("nn", A, B), ("nt", A, B.T.copy()), ("tn", A.T.copy(), B)):
        _, Bd = oracle.gemm(op, x, y)
        np.testing.assert_allclose(Bd, aA @ aB, rtol=1e-13)

    Gall = rng.standard_normal((g.nc, d_out)).astype(np.float32)
    pull = oracle.layer_bwd_pull(g, H[: g.nr], W, Gall, Zprev=Zp)
    aGall = np.abs(Gall.astype(np.float64))
    np.testing.assert_allclose(pull["BT"], M @ aGall, rtol=1e-12)
    np.testing.assert_allclose(pull["BdH"], M @ aGall @ aW.T, rtol=1e-12)
    np.testing.assert_allclose(pull["BdW"], aH[: g.nr].T @ (M @ aGall), rtol=1e-12)

    Z = (3 * rng.standard_normal((g.nr, d_out))).astype(np.float32)
    y = rng.integers(0, d_out, g.nr).astype(np.int32)
    loss, labs, _ = oracle.softmax_xent(Z, y, 0.125)
    Z64 = Z.astype(np.float64)
    lse = np.log(np.exp(Z64 - Z64.max(1, keepdims=True)).sum(1)) + Z64.max(1)
    zy = Z64[np.arange(g.nr), y]
    assert abs(loss - 0.125 * (lse - zy).sum()) <= 1e-12 * labs
    # the loss bound: at least the sum of the terms' magnitudes, at most a few times the largest logit per row
    assert 0.125 * np.abs(lse - zy).sum() <= labs * (1 + 1e-12)
    assert labs <= 0.125 * (3 * np.abs(Z64).max(1) + np.log(d_out)).sum() * (1 + 1e-12)
