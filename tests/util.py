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
