"""Named synthetic workloads: graph + features + weights + labels, all seeded.

The graphs stand in for the public graphs of the paper's dataset table (Sec. 5), which
are not available offline; features and labels are random, as in the paper's timing runs.
A workload is a plain dict of numpy arrays:
  n, src, dst            raw directed edge list (duplicates / self-loops possible), int32
  X                      float32 [n, dims[0]], N(0,1)
  W                      list of float32 [dims[k], dims[k+1]], Glorot-uniform
  y                      int32 [n], uniform in [0, dims[-1])
  dims                   layer widths
Nothing here computes any part of the GCN method.
"""
from __future__ import annotations

import numpy as np

from . import graphs, prng

BASE_SEED = 1234


def features(n: int, d: int, seed: int) -> np.ndarray:
    return prng.normal(seed, 20, n * d).reshape(n, d)


def glorot(d_in: int, d_out: int, seed: int, layer: int) -> np.ndarray:
    lim = np.sqrt(6.0 / (d_in + d_out))
    u = prng.uniform01(seed, 30 + layer, 0, d_in * d_out)
    return ((2.0 * u - 1.0) * lim).astype(np.float32).reshape(d_in, d_out)


def labels(n: int, n_classes: int, seed: int) -> np.ndarray:
    return prng.randint(seed, 40, 0, n, n_classes).astype(np.int32)


def _pack(n, src, dst, dims, seed, with_features=True):
    w = {"n": int(n), "src": src, "dst": dst, "dims": list(dims), "seed": seed}
    w["W"] = [glorot(dims[k], dims[k + 1], seed, k) for k in range(len(dims) - 1)]
    w["y"] = labels(n, dims[-1], seed)
    if with_features:
        w["X"] = features(n, dims[0], seed)
    return w


def tiny_er(n: int = 4096, avg_degree: float = 16.0, dims=(64, 16, 8), seed: int = BASE_SEED + 1):
    """Config 1: Erdos-Renyi, n=4096, average degree 16."""
    src, dst = graphs.erdos_renyi(n, avg_degree, seed)
    return _pack(n, src, dst, dims, seed)


def rmat_powerlaw(scale: int = 18, avg_degree: float = 50.0, dims=(128, 128, 16),
                  seed: int = BASE_SEED + 2, n: int | None = None, permute: bool = True):
    """Config 2: R-MAT (0.57, 0.19, 0.19, 0.05), n = 2**scale, average degree 50."""
    n = (1 << scale) if n is None else n
    src, dst = graphs.rmat(scale, n, int(n * avg_degree / 2), seed, permute=permute)
    return _pack(n, src, dst, dims, seed)


def dense_neighbourhood(n: int = 232_965, n_directed_edges: int = 114_615_892, sigma: float = 1.0,
                        dims=(602, 128, 41), seed: int = BASE_SEED + 3):
    """Config 3: the vertex and edge counts of the paper's densest graph (dataset table, last row)."""
    src, dst = graphs.lognormal_chung_lu(n, n_directed_edges, sigma, seed)
    return _pack(n, src, dst, dims, seed)


def sparse_large(n: int = 2_449_029, scale: int = 22, avg_degree: float = 50.5,
                 dims=(100, 256, 256, 47), seed: int = BASE_SEED + 4):
    """Config 4: R-MAT skew at scale 22 cut to n vertices, about 123.7 M directed edges."""
    frac = (n / float(1 << scale)) ** 2          # rough share of samples that survive the cut
    # 0.46: measured share of surviving samples that are new, distinct edges at this size
    src, dst = graphs.rmat(scale, n, int(n * avg_degree / 2 / max(frac, 1e-3) * 0.46), seed)
    return _pack(n, src, dst, dims, seed)


def row_block(n_global: int = 1 << 25, n_rows: int = 1 << 22, n_halo: int = 6 << 20, avg_degree: float = 16.0,
              dims=(128, 128, 32), seed: int = BASE_SEED + 5):
    """Config 5: one processor's row block of a much larger power-law graph (owned rows + halo columns).

    Extra keys: row_lo, row_hi, deg_global (int32 [n]: entries of each halo vertex's row of A + I, drawn from the
    same row-length law as the owned rows; 1 everywhere else, the owned vertices included), table_seed (the
    feature table is workloads.table: every row recomputable).  y has one label per owned row; no X.
    """
    row_lo = (n_global // 4 // 64) * 64
    src, dst, halo_ids = graphs.row_block(n_global, row_lo, n_rows, n_halo, avg_degree, 0.5, seed)
    # degrees of the halo vertices, whose rows other processors hold; owned vertices keep the placeholder 1 (the build
    # counts their rows itself and never reads these entries)
    deg = np.ones(n_global, dtype=np.int32)
    u = prng.uniform01(seed, 11, 0, n_halo)
    raw = np.minimum((1.0 - u) ** (-1.0 / 1.2), 1.0e5)
    deg[halo_ids] = np.maximum(2, np.floor(raw * (avg_degree - 1.0) / raw.mean() + 1.5)).astype(np.int32)
    w = {"n": int(n_global), "src": src, "dst": dst, "dims": list(dims), "seed": seed,
         "row_lo": int(row_lo), "row_hi": int(row_lo + n_rows), "deg_global": deg, "table_seed": seed + 100}
    w["W"] = [glorot(dims[k], dims[k + 1], seed, k) for k in range(len(dims) - 1)]
    w["y"] = labels(n_rows, dims[-1], seed)
    return w


WORKLOADS = {
    "c1_er4096": tiny_er,
    "c2_rmat18": rmat_powerlaw,
    "c3_dense233k": dense_neighbourhood,
    "c4_sparse2m4": sparse_large,
    "c5_block": row_block,
}


def get(name: str, **kw):
    return WORKLOADS[name](**kw)
