"""Seeded synthetic edge lists shaped like the paper's graphs (dataset table, Sec. 5).

Each generator returns a *raw directed edge list* (src, dst) of int32 global vertex ids.
The lists are deliberately not canonical: they may hold duplicate edges and self-loops,
exactly what the CSR build step has to cope with.  No normalisation, degree counting or
any other step of the GCN method happens here.
"""
from __future__ import annotations

import numpy as np

from . import prng


def _symmetrise(u: np.ndarray, v: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    src = np.concatenate([u, v]).astype(np.int32)
    dst = np.concatenate([v, u]).astype(np.int32)
    return src, dst


def erdos_renyi(n: int, avg_degree: float, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """Undirected G(n, p) with p = avg_degree / (n - 1); both directions listed.

    Every unordered pair {u < v} gets one uniform draw (pair k of the row-major upper
    triangle uses draw k), so this is meant for n up to a few tens of thousands.
    """
    p = avg_degree / (n - 1)
    us, vs = [], []
    k = 0
    for u in range(n - 1):
        cnt = n - 1 - u
        hit = np.nonzero(prng.uniform01(seed, 1, k, cnt) < p)[0]
        k += cnt
        if hit.size:
            us.append(np.full(hit.size, u, dtype=np.int64))
            vs.append(hit + (u + 1))
    u = np.concatenate(us) if us else np.zeros(0, np.int64)
    v = np.concatenate(vs) if vs else np.zeros(0, np.int64)
    return _symmetrise(u, v)


def rmat(scale: int, n: int, n_samples: int, seed: int,
         abcd=(0.57, 0.19, 0.19, 0.05), permute: bool = True,
         chunk: int = 1 << 22) -> tuple[np.ndarray, np.ndarray]:
    """R-MAT samples on a 2**scale grid, endpoints >= n rejected, then symmetrised.

    Sample s uses draws s*scale .. s*scale+scale-1 of stream 2 (one per recursion level,
    most significant bit first).  With permute=True vertex ids are relabelled by a seeded
    permutation so that the hubs are not the low ids.  Duplicates and self-loops are kept.
    """
    a, b, c, _ = abcd
    ab, abc = a + b, a + b + c
    us, vs = [], []
    for s0 in range(0, n_samples, chunk):
        s1 = min(n_samples, s0 + chunk)
        m = s1 - s0
        r = prng.uniform01(seed, 2, s0 * scale, m * scale).reshape(m, scale)
        row_bit = (r >= ab)                      # quadrants c, d: lower half
        col_bit = ((r >= a) & (r < ab)) | (r >= abc)   # quadrants b, d: right half
        weights = (1 << np.arange(scale - 1, -1, -1)).astype(np.int64)
        u = row_bit.astype(np.int64) @ weights
        v = col_bit.astype(np.int64) @ weights
        keep = (u < n) & (v < n)
        us.append(u[keep])
        vs.append(v[keep])
    u = np.concatenate(us)
    v = np.concatenate(vs)
    if permute:
        perm = prng.permutation(seed, 3, n)
        u, v = perm[u], perm[v]
    return _symmetrise(u, v)


def lognormal_chung_lu(n: int, n_directed_edges: int, sigma: float, seed: int,
                       chunk: int = 1 << 23) -> tuple[np.ndarray, np.ndarray]:
    """Chung-Lu graph whose expected degrees follow a log-normal law (dense-neighbourhood shape).

    Vertex weights w_i = exp(sigma * N(0,1)); n_directed_edges/2 endpoint pairs are drawn
    with probability proportional to w_u * w_v (inverse-CDF lookup), then symmetrised.
    Duplicates and self-loops are kept, so the canonical edge count ends somewhat below
    n_directed_edges.
    """
    w = np.exp(sigma * prng.normal(seed, 4, n).astype(np.float64))
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    m = n_directed_edges // 2
    us, vs = [], []
    for s0 in range(0, m, chunk):
        s1 = min(m, s0 + chunk)
        r = prng.uniform01(seed, 5, 2 * s0, 2 * (s1 - s0))
        us.append(np.minimum(np.searchsorted(cdf, r[0::2], side="right"), n - 1).astype(np.int32))
        vs.append(np.minimum(np.searchsorted(cdf, r[1::2], side="right"), n - 1).astype(np.int32))
    return _symmetrise(np.concatenate(us), np.concatenate(vs))


def row_block(n_global: int, row_lo: int, n_rows: int, n_halo: int, avg_degree: float,
              p_local: float, seed: int, chunk: int = 1 << 22):
    """One processor's row block of a much larger power-law graph, synthesised directly.

    Returns (src, dst, deg_global_sparse) where src lies in [row_lo, row_lo + n_rows),
    dst is a global id, and the block's non-owned columns are drawn from a fixed set of
    n_halo distinct global ids with a power-law popularity.  Row lengths follow a discrete
    power law scaled to the requested mean.  Each entry is local with probability p_local.
    """
    # row lengths: Pareto-like, mean avg_degree (minus the self-loop the build adds)
    u = prng.uniform01(seed, 6, 0, n_rows)
    alpha = 2.2
    raw = (1.0 - u) ** (-1.0 / (alpha - 1.0))            # >= 1, heavy tail
    raw = np.minimum(raw, 1.0e5)
    lens = np.maximum(1, np.floor(raw * (avg_degree - 1.0) / raw.mean() + 0.5)).astype(np.int64)
    total = int(lens.sum())
    src = np.repeat(np.arange(row_lo, row_lo + n_rows, dtype=np.int64), lens)
    # halo id set: n_halo distinct non-owned ids, spread over the global range
    stride = (n_global - n_rows) // n_halo
    assert stride >= 1
    base = np.arange(n_halo, dtype=np.int64) * stride + prng.randint(seed, 7, 0, n_halo, stride)
    halo_ids = np.where(base >= row_lo, base + n_rows, base)      # skip the owned range
    rank_of = prng.permutation(seed, 8, n_halo)                   # popularity rank -> id slot
    dst = np.empty(total, dtype=np.int64)
    for e0 in range(0, total, chunk):
        e1 = min(total, e0 + chunk)
        m = e1 - e0
        is_local = prng.uniform01(seed, 9, e0, m) < p_local
        r = prng.uniform01(seed, 10, e0, m)
        loc = row_lo + np.minimum((r ** 1.5 * n_rows).astype(np.int64), n_rows - 1)   # mildly skewed
        pop = np.minimum((r ** 3.0 * n_halo).astype(np.int64), n_halo - 1)            # strongly skewed
        dst[e0:e1] = np.where(is_local, loc, halo_ids[rank_of[pop]])
    return src.astype(np.int32), dst.astype(np.int32), halo_ids
