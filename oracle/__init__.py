"""CPU oracle for the GCN layer path -- TEST INFRASTRUCTURE, not product code.

Thin ctypes/numpy wrapper over ``gcn_oracle.c`` (plain C, fp64 accumulation, written from
the paper's definitions).  Only the tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; the GPU library never does, and this package never imports
the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gcn_oracle.c")
_LIB = os.path.join(_HERE, "libgcn_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: fp64 sums stay in source order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


class _Graph(C.Structure):
    _fields_ = [("nr", C.c_int64), ("nh", C.c_int64), ("nnz", C.c_int64),
                ("rowptr", C.POINTER(C.c_int64)), ("col", C.POINTER(C.c_int32)),
                ("val", C.POINTER(C.c_float)), ("val64", C.POINTER(C.c_double)),
                ("deg", C.POINTER(C.c_int32)), ("halo_gid", C.POINTER(C.c_int32)),
                ("colptr", C.POINTER(C.c_int64)), ("rowidx", C.POINTER(C.c_int32)),
                ("val_t", C.POINTER(C.c_float))]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_graph_build.restype = C.c_int
        _lib.orc_gather.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


@dataclass
class Graph:
    nr: int
    nh: int
    nnz: int
    rowptr: np.ndarray
    col: np.ndarray
    val: np.ndarray
    val64: np.ndarray
    deg: np.ndarray
    halo_gid: np.ndarray
    colptr: np.ndarray
    rowidx: np.ndarray
    val_t: np.ndarray

    @property
    def nc(self) -> int:
        return self.nr + self.nh


def graph_build(src, dst, n_global, row_lo=0, row_hi=None, deg_global=None) -> Graph:
    """Normalised adjacency block in CSR + CSC + halo list (see gcn_oracle.c)."""
    row_hi = n_global if row_hi is None else row_hi
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    dg = None if deg_global is None else np.ascontiguousarray(deg_global, dtype=np.int32)
    g = _Graph()
    rc = lib().orc_graph_build(_p(src, C.c_int32), _p(dst, C.c_int32), C.c_int64(src.size),
                               C.c_int64(n_global), C.c_int64(row_lo), C.c_int64(row_hi),
                               _p(dg, C.c_int32), C.byref(g))
    if rc != 0:
        raise ValueError("oracle graph_build: invalid input")
    nr, nh, nnz = g.nr, g.nh, g.nnz

    def take(ptr, n, dt):
        return np.ctypeslib.as_array(ptr, shape=(max(n, 1),))[:n].astype(dt, copy=True)

    out = Graph(nr, nh, nnz,
                take(g.rowptr, nr + 1, np.int64), take(g.col, nnz, np.int32),
                take(g.val, nnz, np.float32), take(g.val64, nnz, np.float64),
                take(g.deg, nr, np.int32), take(g.halo_gid, nh, np.int32),
                take(g.colptr, nr + nh + 1, np.int64), take(g.rowidx, nnz, np.int32),
                take(g.val_t, nnz, np.float32))
    lib().orc_graph_free(C.byref(g))
    return out


def spmm(ptr, idx, val, X, rows=None, want_bound=True):
    """Y = A X (fp64) and the bound sum |A||X|; rows=None -> all rows of A, else only those."""
    X = _f32(X)
    ptr = np.ascontiguousarray(ptr, dtype=np.int64)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = _f32(val)
    d = X.shape[1]
    if rows is None:
        n, rp = ptr.size - 1, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, rp = rows.size, _p(rows, C.c_int64)
    Y = np.empty((n, d), dtype=np.float64)
    B = np.empty((n, d), dtype=np.float64) if want_bound else None
    lib().orc_spmm(_p(ptr, C.c_int64), _p(idx, C.c_int32), _p(val, C.c_float), C.c_int64(n), rp,
                   _p(X, C.c_float), C.c_int64(X.shape[1]), C.c_int64(d), _p(Y, C.c_double),
                   _p(B, C.c_double))
    return Y, B


def gemm(op: str, A, B):
    """op in {'nn','nt','tn'}: A B, A B^T, A^T B in fp64 with the absolute-value bound."""
    A, B = _f32(A), _f32(B)
    code = {"nn": 0, "nt": 1, "tn": 2}[op]
    if code == 0:
        M, K = A.shape; N = B.shape[1]; assert B.shape[0] == K
    elif code == 1:
        M, K = A.shape; N = B.shape[0]; assert B.shape[1] == K
    else:
        K, M = A.shape; N = B.shape[1]; assert B.shape[0] == K
    Cm = np.empty((M, N), dtype=np.float64)
    Bd = np.empty((M, N), dtype=np.float64)
    lib().orc_gemm(C.c_int(code), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(A, C.c_float),
                   C.c_int64(A.shape[1]), _p(B, C.c_float), C.c_int64(B.shape[1]),
                   _p(Cm, C.c_double), _p(Bd, C.c_double))
    return Cm, Bd


def gemm_dd(op: str, A, B):
    """The same products for fp64 operands (no rounding of a factor that is itself an fp64 result)."""
    A = np.ascontiguousarray(A, dtype=np.float64); B = np.ascontiguousarray(B, dtype=np.float64)
    code = {"nn": 0, "nt": 1, "tn": 2}[op]
    if code == 0:
        M, K = A.shape; N = B.shape[1]; assert B.shape[0] == K
    elif code == 1:
        M, K = A.shape; N = B.shape[0]; assert B.shape[1] == K
    else:
        K, M = A.shape; N = B.shape[1]; assert B.shape[0] == K
    Cm = np.empty((M, N), dtype=np.float64)
    lib().orc_gemm_dd(C.c_int(code), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(A, C.c_double),
                      C.c_int64(A.shape[1]), _p(B, C.c_double), C.c_int64(B.shape[1]), _p(Cm, C.c_double))
    return Cm


def layer_fwd(g: Graph, H, W, bias=None, act="relu"):
    """Returns dict(AH, Z, Hout, Bz), all fp64."""
    H, W = _f32(H), _f32(W)
    assert H.shape[0] == g.nc and W.shape[0] == H.shape[1]
    d_in, d_out = W.shape
    b = None if bias is None else _f32(bias)
    AH = np.empty((g.nr, d_in)); Z = np.empty((g.nr, d_out))
    Ho = np.empty((g.nr, d_out)); Bz = np.empty((g.nr, d_out))
    lib().orc_layer_fwd(_p(g.rowptr, C.c_int64), _p(g.col, C.c_int32), _p(g.val, C.c_float),
                        C.c_int64(g.nr), C.c_int64(g.nc), _p(H, C.c_float), C.c_int64(d_in),
                        _p(W, C.c_float), _p(b, C.c_float), C.c_int64(d_in), C.c_int64(d_out),
                        C.c_int(1 if act == "relu" else 0), _p(AH, C.c_double), _p(Z, C.c_double),
                        _p(Ho, C.c_double), _p(Bz, C.c_double))
    return {"AH": AH, "Z": Z, "Hout": Ho, "Bz": Bz}


def layer_bwd(g: Graph, H, W, G, Zprev=None, want_dH=True, want_dbias=False):
    """Returns dict(dW, BdW, dH, BdH, dbias, Bdb), fp64 (dH/dbias None when not requested)."""
    H, W, G = _f32(H), _f32(W), _f32(G)
    d_in, d_out = W.shape
    assert H.shape == (g.nc, d_in) and G.shape == (g.nr, d_out)
    Zp = None if Zprev is None else _f32(Zprev)
    dW = np.empty((d_in, d_out)); BdW = np.empty((d_in, d_out))
    dH = np.empty((g.nc, d_in)) if want_dH else None
    BdH = np.empty((g.nc, d_in)) if want_dH else None
    db = np.empty(d_out) if want_dbias else None
    Bdb = np.empty(d_out) if want_dbias else None
    lib().orc_layer_bwd(_p(g.rowptr, C.c_int64), _p(g.col, C.c_int32), _p(g.val, C.c_float),
                        _p(g.colptr, C.c_int64), _p(g.rowidx, C.c_int32), _p(g.val_t, C.c_float),
                        C.c_int64(g.nr), C.c_int64(g.nc), _p(H, C.c_float), C.c_int64(d_in),
                        _p(W, C.c_float), _p(G, C.c_float), C.c_int64(d_out),
                        _p(Zp, C.c_float), C.c_int64(d_in), C.c_int64(d_in), C.c_int64(d_out),
                        _p(dW, C.c_double), _p(BdW, C.c_double), _p(dH, C.c_double),
                        _p(BdH, C.c_double), _p(db, C.c_double), _p(Bdb, C.c_double))
    return {"dW": dW, "BdW": BdW, "dH": dH, "BdH": BdH, "dbias": db, "Bdb": Bdb}


def layer_bwd_pull(g: Graph, H_owned, W, G_all, Zprev=None):
    """Backward pass of one layer as Algorithm 2 (Sec. 4.2) states it for processor m, steps in its order:
    T = A_m [G_m; G_halo] (the by-product), S = T W^T, G^(k-1)_m = S (.) [Zprev > 0], dW_m = H_m^T T.
    Returns dict(T, BT, dH, BdH, dW, BdW) in fp64; B* are the same sums over absolute values."""
    H_owned, W, G_all = _f32(H_owned), _f32(W), _f32(G_all)
    d_in, d_out = W.shape
    assert H_owned.shape == (g.nr, d_in) and G_all.shape == (g.nc, d_out)
    T, BT = spmm(g.rowptr, g.col, g.val, G_all)
    W64, H64 = W.astype(np.float64), H_owned.astype(np.float64)
    S, BS = gemm_dd("nt", T, W64), gemm_dd("nt", BT, np.abs(W64))
    if Zprev is not None:
        keep = _f32(Zprev) > 0
        assert keep.shape == S.shape
        S = np.where(keep, S, 0.0)
    return {"T": T, "BT": BT, "dH": S, "BdH": BS, "dW": gemm_dd("tn", H64, T), "BdW": gemm_dd("tn", np.abs(H64), BT)}


def softmax_xent(Z, y, scale):
    """Returns (loss, loss_bound, G) in fp64."""
    Z = _f32(Z)
    y = np.ascontiguousarray(y, dtype=np.int32)
    nr, Cn = Z.shape
    G = np.empty((nr, Cn), dtype=np.float64)
    loss = C.c_double(0.0); labs = C.c_double(0.0)
    lib().orc_softmax_xent(_p(Z, C.c_float), C.c_int64(Cn), C.c_int64(nr), C.c_int64(Cn),
                           _p(y, C.c_int32), C.c_double(scale), C.byref(loss), C.byref(labs),
                           _p(G, C.c_double))
    return loss.value, labs.value, G


def gather(table, idx):
    table = _f32(table)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    out = np.empty((idx.size, table.shape[1]), dtype=np.float32)
    rc = lib().orc_gather(_p(table, C.c_float), C.c_int64(table.shape[1]), C.c_int64(table.shape[0]),
                          C.c_int64(table.shape[1]), _p(idx, C.c_int32), C.c_int64(idx.size),
                          _p(out, C.c_float), C.c_int64(table.shape[1]))
    if rc != 0:
        raise ValueError("oracle gather: index out of range")
    return out


def sgd_update(W, dW, lr):
    """Gradient-descent step W - lr * dW (Sec. 3.1, the weight update), fp64 arithmetic, returned as fp32."""
    return (np.asarray(W, dtype=np.float64) - float(lr) * np.asarray(dW, dtype=np.float64)).astype(np.float32)


def train(g: Graph, X, Ws, y, lr, epochs, scale=None):
    """Full-batch training of an L-layer GCN (Algorithm 1 forward, Algorithm 2 backward and update, on one
    block): ReLU on all layers but the last, softmax cross-entropy on the last pre-activation.  Every stored
    array (layer outputs, gradients, weights) is rounded to fp32 between steps, as the arrays of an fp32
    implementation are; all sums are fp64.  Returns (losses per epoch before the update, final weights)."""
    Ws = [np.asarray(W, dtype=np.float32).copy() for W in Ws]
    L = len(Ws)
    scale = 1.0 / g.nr if scale is None else scale
    assert g.nh == 0, "training loop needs a whole graph (halo rows come from other processors)"
    losses = []
    for _ in range(epochs):
        H = [_f32(X)]
        for k in range(L):
            f = layer_fwd(g, H[k], Ws[k], act="none" if k == L - 1 else "relu")
            H.append((f["Z"] if k == L - 1 else f["Hout"]).astype(np.float32))
        loss, _, G = softmax_xent(H[L], y, scale)
        losses.append(loss)
        G = G.astype(np.float32)
        dWs = [None] * L
        for k in range(L - 1, -1, -1):
            b = layer_bwd(g, H[k], Ws[k], G, Zprev=H[k][: g.nr] if k > 0 else None, want_dH=k > 0)
            dWs[k] = b["dW"]
            if k > 0:
                G = b["dH"][: g.nr].astype(np.float32)
        Ws = [sgd_update(Ws[k], dWs[k], lr) for k in range(L)]
    return losses, Ws


def partition_stats(colptr, rowidx, rowptr, part, p):
    """Communication figures of a 1D row partition under the column-net hypergraph model (Sec. 4.3.2): net n_j
    joins the rows with a stored entry in column j; the part that owns vertex j sends row j once to every other
    part of the net's connectivity set.  Plain loops over the nets, integers only.

    part[i] in [0, p) for every vertex.  Returns a dict of
      volume      sum_j (lambda(n_j) - 1): rows sent per sparse product (the paper's total, without its constant
                  factors 2 and cost(n_j))
      cut_entries stored entries (i, j) with part[i] != part[j] (what the graph model charges)
      load[m]     sum of w(v_i) = stored entries in the rows of part m
      send_rows[m], recv_rows[m]   rows part m sends / receives per product
      send_msgs[m], recv_msgs[m]   number of parts it sends to / receives from
    """
    colptr = np.asarray(colptr, np.int64); rowidx = np.asarray(rowidx, np.int64)
    rowptr = np.asarray(rowptr, np.int64); part = np.asarray(part, np.int64)
    n = colptr.size - 1
    assert part.size == n and rowptr.size == n + 1 and part.min(initial=0) >= 0 and part.max(initial=0) < p
    send_rows = np.zeros(p, np.int64); recv_rows = np.zeros(p, np.int64)
    pairs = set()
    cut = 0
    for j in range(n):
        pins = rowidx[colptr[j]:colptr[j + 1]]
        owner = int(part[j])
        cut += int(np.count_nonzero(part[pins] != owner))
        for q in set(part[pins].tolist()) - {owner}:          # connectivity set minus the owner
            send_rows[owner] += 1
            recv_rows[q] += 1
            pairs.add((owner, q))
    send_msgs = np.zeros(p, np.int64); recv_msgs = np.zeros(p, np.int64)
    for m, q in pairs:
        send_msgs[m] += 1
        recv_msgs[q] += 1
    load = np.zeros(p, np.int64)
    for i in range(n):
        load[part[i]] += rowptr[i + 1] - rowptr[i]
    return {"volume": int(send_rows.sum()), "cut_entries": cut, "load": load, "send_rows": send_rows,
            "recv_rows": recv_rows, "send_msgs": send_msgs, "recv_msgs": recv_msgs}


def induced_edges(src, dst, n, vertices):
    """Edge list of the subgraph induced by a vertex list, in the subgraph's numbering (Sec. 4.3.3: a mini-batch
    is G' = (V', E'), V' a subset of V and E' the edges of E between vertices of V'): vertex k of G' is
    vertices[k].  graph_build on the result gives the subgraph's own normalised adjacency."""
    src = np.asarray(src, np.int64); dst = np.asarray(dst, np.int64); vertices = np.asarray(vertices, np.int64)
    assert np.unique(vertices).size == vertices.size and vertices.min() >= 0 and vertices.max() < n
    number = np.full(n, -1, np.int64)
    number[vertices] = np.arange(vertices.size)
    keep = (number[src] >= 0) & (number[dst] >= 0)
    return number[src[keep]].astype(np.int32), number[dst[keep]].astype(np.int32)
