"""A huge feature table whose every entry is a pure function of (row, column, seed).

It stands in for the feature rows that live on other processors (or on the host): any row can be
recomputed on the CPU for a check without materialising the table there.  Values are multiples of
2^-23 in [-1, 1): exactly representable in fp32 (and produced with integer arithmetic only, so the
numpy and the torch evaluation agree bit for bit).  No GCN arithmetic here.
"""
from __future__ import annotations

import numpy as np

_A, _B, _C = 0x9E3779B1, 0x85EBCA77, 0xC2B2AE3D
_MASK32 = 0xFFFFFFFF


def table_rows(rows, d: int, seed: int) -> np.ndarray:
    """float32 [len(rows), d]: the table rows with the given (global) row ids."""
    r = np.asarray(rows, dtype=np.int64).reshape(-1, 1)
    c = np.arange(d, dtype=np.int64).reshape(1, -1)
    h = (r * _A + c * _B + (seed * _C & _MASK32)) & _MASK32
    h = (h ^ (h >> 15)) * 0x2C1B3C6D & _MASK32
    h = h ^ (h >> 12)
    return ((h >> 8).astype(np.float32) * np.float32(2.0 ** -23) - np.float32(1.0)).astype(np.float32)


def fill_table_torch(table, seed: int, device, chunk_rows: int = 1 << 20):
    """Fills a (pinned host or device) torch float32 tensor [n, d] with the same values, evaluating the
    integer hash on `device` chunk by chunk."""
    import torch
    n, d = table.shape
    c = torch.arange(d, dtype=torch.int64, device=device).view(1, -1)
    s = seed * _C & _MASK32
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        r = torch.arange(r0, r1, dtype=torch.int64, device=device).view(-1, 1)
        h = (r * _A + c * _B + s) & _MASK32
        h = ((h ^ (h >> 15)) * 0x2C1B3C6D) & _MASK32
        h = h ^ (h >> 12)
        v = (h >> 8).to(torch.float32) * (2.0 ** -23) - 1.0
        table[r0:r1].copy_(v, non_blocking=False)
    return table
