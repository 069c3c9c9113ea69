"""Helpers shared by the GPU parity tests."""
from __future__ import annotations

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
    return float(ratio)
