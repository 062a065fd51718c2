"""Helpers shared by the GPU parity tests: run the oracle's phase functions over rows in a
thread pool (the oracle itself stays single-threaded per call) and compare states."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import List, Tuple

import numpy as np

import oracle

POOL = ThreadPoolExecutor(max_workers=16)

# Tolerances of the parity bar: max relative error of fp32 state after one step / after a chain.
TOL_STEP = 1e-5
TOL_CHAIN = 1e-4


def oracle_step_rows(g: np.ndarray, x: np.ndarray, e: np.ndarray, wc: str, sc: str, lr: float,
                     wk: int = 0, sk: int = 0, rng: Tuple[int, int] = (0, 0)):
    """Algorithm 1's compressed iteration assembled from the oracle's phases, with the per-worker
    phases running concurrently.  x and e are updated in place.  rng = (seed, draw) names the
    iteration's random-k draws (worker i draws with row i, the server with row N).  Returns
    (worker descs, server desc, v, p, P)."""
    N, d = g.shape
    res = list(POOL.map(lambda i: oracle.compress(wc, g[i], wk, rng=(rng[0], rng[1], i)), range(N)))
    P = np.stack([r[0] for r in res]) if N > 1 else res[0][0][None, :]
    wdesc = [r[1] for r in res]
    v = oracle.server_average(P, e)
    p, sdesc = oracle.compress(sc, v, sk, rng=(rng[0], rng[1], N))
    e[:] = oracle.error_update(v, p)
    list(POOL.map(lambda i: oracle.worker_update(g[i], P[i], p, lr, x[i]), range(N)))
    return wdesc, sdesc, v, p, P


def rel_err(a: np.ndarray, ref: np.ndarray) -> float:
    """max_j |a_j - ref_j| / max(|ref_j|, rms(ref)) -- plain relative error is meaningless where
    ref passes through zero."""
    a64, r64 = a.astype(np.float64).ravel(), ref.astype(np.float64).ravel()
    if a64.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r64 * r64)))
    den = np.maximum(np.abs(r64), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(a64 - r64) / den))


def sign_bits(v: np.ndarray) -> np.ndarray:
    return v < 0


def topk_mask(v: np.ndarray, tau: int, cutoff: int) -> np.ndarray:
    key = v.view(np.uint32) & np.uint32(0x7FFFFFFF)
    idx = np.arange(v.size, dtype=np.int64)
    return (key > np.uint32(tau)) | ((key == np.uint32(tau)) & (idx <= cutoff))


def bit_equal(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))
