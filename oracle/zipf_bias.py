"""Calibration of the router's second bias so that expert popularity follows Zipf(s).

TEST INFRASTRUCTURE ONLY (part of the oracle side).  The skewed benchmark workload asks for
top-k selection shares q_r ~ r^-s over the experts (expert 0 the most popular).  The closed
form b = log q does not give that under top-k selection of nearly deterministic logits, so
the bias is found by fixed-point iteration on the fp64 oracle router: measure the selection
shares f on a sample of slices, move b by eta * (log q - log f), repeat.  The result is just
an input tensor (rounded to the storage dtype) that oracle and GPU path both consume.
"""
from __future__ import annotations

import numpy as np

from . import route


def zipf_shares(E: int, s: float) -> np.ndarray:
    q = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    return q / q.sum()


def selection_shares(idx: np.ndarray, E: int) -> np.ndarray:
    return np.bincount(idx.reshape(-1), minlength=E).astype(np.float64) / idx.size


def calibrate_zipf_bias(x, Wr1, br1, Wr2, k: int, s: float, round_fn, iters: int = 200,
                        eta: float = 0.05, tol: float = 0.02):
    """Return (bias[E] float32 storage-rounded, achieved shares, iterations used)."""
    E = Wr2.shape[1]
    q = zipf_shares(E, s)
    r = route(x, Wr1, br1, Wr2, np.zeros(E), k, want_logits=True)
    b = -r["logits"].mean(axis=0)  # start from equalised mean logits
    best = None
    for it in range(iters):
        bs = round_fn(b.astype(np.float32))
        f = selection_shares(route(x, Wr1, br1, Wr2, bs, k)["idx"], E)
        err = np.max(np.abs(f / q - 1.0))
        if best is None or err < best[0]:
            best = (err, bs.copy(), f.copy(), it)
        if err < tol:
            break
        b = b + eta * (np.log(q) - np.log(np.maximum(f, 1e-6)))
    return best[1], best[2], best[3], best[0]
