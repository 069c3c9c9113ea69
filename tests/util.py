"""Helpers shared by the GPU parity tests."""
from __future__ import annotations

import os
import sys

import numpy as np

TOL_F32 = 1e-5     # per-element: |gpu - oracle| <= TOL * sum of |terms|
TOL_BF16 = 2e-2


def say(msg: str):
    """Name the case before the GPU step runs, flushed, so a fault can be attributed."""
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def check_bound(gpu, ref, bound, tol=TOL_F32, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bound = np.asarray(bound, dtype=np.float64)
    assert gpu.shape == ref.shape == bound.shape, (what, gpu.shape, ref.shape, bound.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output"
    err = np.abs(gpu - ref)
    lim = tol * bound
    bad = err > lim
    if bad.any():
        k = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements outside {tol:g}*sum|terms|; worst at {k}: "
                             f"gpu={gpu[k]!r} ref={ref[k]!r} err={err[k]:.3e} limit={lim[k]:.3e}")
    ratio = np.max(err / np.maximum(lim, 1e-300)) if err.size else 0.0
    log = os.environ.get("GCN_TEST_RATIO_LOG")      # optional record of how much of each tolerance was used
    if log:
        with open(log, "a") as f:
            f.write(f"{tol:g}\t{float(ratio):.4f}\t{what}\n")
    return float(ratio)


def bf16_round(a):
    """fp32 array -> nearest bf16 value (ties to even), returned as fp32. Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def to_dev(a, dev, bf16=False):
    """numpy -> GPU tensor; with bf16=True the (already bf16-representable) values are stored as bf16."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    return t.to(torch.bfloat16) if bf16 else t


def to_np(t):
    """GPU tensor -> numpy (bf16 widened to fp32 exactly)."""
    import torch
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.detach().cpu().numpy()


def hub_graph(n, n_hubs, avg_degree, seed):
    """Undirected edge list with a few very long rows: hub h is linked to every (h+2)-th vertex."""
    rng = np.random.default_rng(seed)
    m = int(n * avg_degree / 2)
    u = rng.integers(0, n, m); v = rng.integers(0, n, m)
    us, vs = [u], [v]
    for h in range(n_hubs):
        nb = np.arange(0, n, h + 1)
        us.append(np.full(nb.size, h)); vs.append(nb)
    u = np.concatenate(us); v = np.concatenate(vs)
    return np.concatenate([u, v]).astype(np.int32), np.concatenate([v, u]).astype(np.int32)


def sample_rows(og, n_random, seed, n_longest=40):
    """Row sample for full-size checks: the longest rows, a few of the shortest, the first and the last, random ones."""
    rng = np.random.default_rng(seed)
    order = np.argsort(-og.deg.astype(np.int64), kind="stable")
    return np.unique(np.concatenate([order[:n_longest], order[-5:], rng.integers(0, og.nr, n_random),
                                     [0, og.nr - 1]])).astype(np.int64)


def check_epoch_sampled(ep, w, og, rows, tol, dw_cols=6, seed=11, log=None):
    """Every call of one bench.Epoch pass (push form) against the oracle at a size where the oracle cannot redo
    whole layers: each call is recomputed from the GPU's own inputs of that call (copied back), on

      * the sampled output rows `rows` of every row-wise result (layer outputs, saved A^ H, gradients handed down,
        for a block also sampled halo rows of dH), through oracle.spmm(rows=...) and the oracle's fp64 products;
      * the loss and every element of the output gradient;
      * every element of the last layer's dW and `dw_cols` sampled columns of every other dW.  A column c of
        dW = (A^ H)^T G is H^T (A^T G[:, c]): the oracle's sparse product of the transposed arrays with those
        columns of G, then a dense fp64 product (numpy, one step of the definition) over all rows.

    Bounds are the same sums over absolute values; tolerance tol * bound per element."""
    import oracle
    import numpy as _np
    say = log or (lambda m: None)
    L = len(w["W"])
    nr = og.nr
    W64 = [m.astype(_np.float64) for m in w["W"]]
    Hs = [to_np(ep.H[k]) for k in range(L)]
    for k in range(L):
        last = k == L - 1
        say(f"forward layer {k}: {rows.size} sampled rows")
        AH, BAH = oracle.spmm(og.rowptr, og.col, og.val, Hs[k], rows=rows)
        Z, B = oracle.gemm_dd("nn", AH, W64[k]), oracle.gemm_dd("nn", BAH, _np.abs(W64[k]))
        got = to_np((ep.Zlast if last else ep.H[k + 1])[rows])
        check_bound(got, Z if last else _np.maximum(Z, 0.0), B, tol, f"layer {k} output rows")
        if ep.AH[k] is not None:
            check_bound(to_np(ep.AH[k][rows]), AH, BAH, tol, f"layer {k} saved A^ H rows")
    Zl = to_np(ep.Zlast)
    loss, labs, G = oracle.softmax_xent(Zl, w["y"], 1.0 / nr)
    assert abs(float(ep.loss.item()) - loss) <= TOL_F32 * max(labs, _np.abs(Zl).max() * 3), "loss"
    onehot = _np.zeros_like(G); onehot[_np.arange(nr), w["y"]] = 1.0 / nr
    check_bound(to_np(ep.G[L - 1]), G, G + 2 * onehot, tol, "output gradient")
    del G, onehot, Zl
    rng = _np.random.default_rng(seed)
    for k in range(L - 1, -1, -1):
        Gk = to_np(ep.G[k])
        d_out = Gk.shape[1]
        cols = _np.arange(d_out) if k == L - 1 else _np.unique(_np.concatenate([[0, d_out - 1], rng.integers(0, d_out, dw_cols)]))
        say(f"backward layer {k}: dW columns {cols.size} of {d_out}")
        Gc = _np.ascontiguousarray(Gk[:, cols])
        T, BT = oracle.spmm(og.colptr, og.rowidx, og.val_t, Gc)          # [nc, |cols|]
        H64 = Hs[k].astype(_np.float64)
        dWc, BdWc = H64.T @ T, _np.abs(H64).T @ BT
        del H64, T, BT
        check_bound(to_np(ep.dW[k])[:, cols], dWc, BdWc, tol, f"dW of layer {k}")
        if k > 0:
            lc = rows if og.nh == 0 else _np.unique(_np.concatenate([rows, nr + _np.arange(0, og.nh, max(1, og.nh // 400))]))
            T, BT = oracle.spmm(og.colptr, og.rowidx, og.val_t, Gk, rows=lc)
            S, BS = oracle.gemm_dd("nt", T, W64[k]), oracle.gemm_dd("nt", BT, _np.abs(W64[k]))
            own = lc < nr
            S[own] = _np.where(Hs[k][lc[own]] > 0, S[own], 0.0)
            check_bound(to_np(ep.D[k - 1][lc]), S, BS, tol, f"gradient handed to layer {k - 1} (rows)")
        del Gk
