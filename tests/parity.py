"""Acceptance rules for comparing the HIP path with the CPU oracle.

Floating point: |g - o| <= tol * max(|o|, S) with S = max(1, RMS of the oracle's
valid predictions on the checked set); tol = 1e-5 for the fp32 path.
Top-k: with o_k the oracle's k-th value and band = tol * max(|o_k|, S):
every oracle index whose value is below o_k - band must be in the GPU set,
every GPU index must be valid with oracle value <= o_k + band, the sizes are
equal, there are no duplicates, the GPU list is sorted by (value, index), and
GPU values match the oracle's values at the same indices within tol.
"""
from __future__ import annotations

import numpy as np

TOL_FP32 = 1e-5


def scale_of(o_valid: np.ndarray) -> float:
    if len(o_valid) == 0:
        return 1.0
    return max(1.0, float(np.sqrt(np.mean(o_valid.astype(np.float64) ** 2))))


def check_predictions(g: np.ndarray, o: np.ndarray, valid: np.ndarray, tol: float = TOL_FP32):
    """g, o: fp32 arrays over the same indices; valid: oracle mask (bool).
    Returns (worst scaled error / tol, worst pure relative error)."""
    valid = valid.astype(bool)
    assert np.all(np.isposinf(g[~valid])), "invalid configurations must be +inf"
    assert np.all(np.isfinite(g[valid])), "valid predictions must be finite"
    if not valid.any():
        return 0.0, 0.0
    gv = g[valid].astype(np.float64)
    ov = o[valid].astype(np.float64)
    S = scale_of(ov)
    err = np.abs(gv - ov) / np.maximum(np.abs(ov), S)
    worst = float(err.max())
    rel = float((np.abs(gv - ov) / np.maximum(np.abs(ov), 1e-30)).max())
    assert worst <= tol, f"prediction error {worst:.3e} > {tol:.1e} (pure relative worst {rel:.3e})"
    return worst / tol, rel


def check_topk(g_vals, g_idx, o_all, valid_all, index_base: int, k: int, tol: float = TOL_FP32):
    """g_vals/g_idx: GPU result (ascending).  o_all/valid_all: oracle predictions
    and mask for every index of the swept range(s) concatenated, where entry t
    is configuration index_base + t."""
    valid_all = valid_all.astype(bool)
    n_valid = int(valid_all.sum())
    assert len(g_idx) == min(k, n_valid), f"n_found {len(g_idx)} != {min(k, n_valid)}"
    if len(g_idx) == 0:
        return
    g_idx = g_idx.astype(np.int64)
    assert len(np.unique(g_idx)) == len(g_idx), "duplicate indices"
    t = g_idx - index_base
    assert np.all((t >= 0) & (t < len(o_all))), "index outside the swept range"
    assert np.all(valid_all[t]), "an invalid configuration was returned"
    # sorted by (value, index)
    gv = g_vals.astype(np.float64)
    order_ok = (gv[1:] > gv[:-1]) | ((gv[1:] == gv[:-1]) & (g_idx[1:] > g_idx[:-1]))
    assert np.all(order_ok), "GPU list is not sorted by (value, index)"
    ov = o_all[valid_all].astype(np.float64)
    S = scale_of(ov)
    # values at the same indices
    o_at = o_all[t].astype(np.float64)
    err = np.abs(gv - o_at) / np.maximum(np.abs(o_at), S)
    assert float(err.max()) <= tol, f"top-k value error {float(err.max()):.3e}"
    # band rule around the oracle's k-th value
    kk = len(g_idx)
    o_k = np.partition(ov, kk - 1)[kk - 1]       # the oracle's k-th smallest value
    band = tol * max(abs(o_k), S)
    assert np.all(o_at <= o_k + band), "GPU returned a configuration above the k-th value band"
    must = np.nonzero(valid_all & (o_all.astype(np.float64) < o_k - band))[0] + index_base
    missing = np.setdiff1d(must, g_idx)
    assert len(missing) == 0, f"{len(missing)} configurations clearly below the k-th value are missing"
