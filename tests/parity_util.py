"""Shared helpers for the GPU parity tests: the comparison rules only.
(No method arithmetic: expected values always come from `oracle`.)"""
from __future__ import annotations

import numpy as np
import torch

REL_MARGIN = 1e-4          # k-th / (k+1)-th score margin above which indices must match exactly
TOL = {torch.float32: dict(max_abs=1e-4, mean_abs=1e-4),
       torch.bfloat16: dict(max_abs=2e-2, mean_abs=1e-2)}


def units(t: torch.Tensor) -> torch.Tensor:
    """[S,H,rows,d] -> [S*H,rows,d] on the CPU."""
    return t.detach().cpu().reshape(t.shape[0] * t.shape[1], *t.shape[2:])


def check_indices(gpu_idx: np.ndarray, scores: np.ndarray, keep: int, oracle_idx: np.ndarray):
    """Index rule for one unit.  scores: the oracle's fp64 scores (all > 0).
    If the relative gap between the keep-th and (keep+1)-th largest exceeds
    REL_MARGIN the GPU list must equal the oracle's; otherwise it must be a valid
    choice inside the near-tie band.  Returns 'exact' or 'band'."""
    gpu_idx = np.asarray(gpu_idx)
    n = len(scores)
    assert gpu_idx.shape == (keep,)
    assert np.all(np.diff(gpu_idx) > 0), "indices must be strictly ascending (no duplicates)"
    if keep:
        assert gpu_idx[0] >= 0 and gpu_idx[-1] < n
    if keep == 0 or keep == n:
        assert np.array_equal(gpu_idx, oracle_idx)
        return "exact"
    order = np.sort(scores)[::-1]
    a, b = order[keep - 1], order[keep]
    if a > 0 and (a - b) / a > REL_MARGIN:
        assert np.array_equal(gpu_idx, oracle_idx), "indices differ although the margin is wide"
        return "exact"
    chosen = np.zeros(n, dtype=bool); chosen[gpu_idx] = True
    must = scores > a * (1 + REL_MARGIN)
    may = scores >= a * (1 - REL_MARGIN)
    assert np.all(chosen[must]), "a clearly-above-threshold token was dropped"
    assert np.all(may[chosen]), "a clearly-below-threshold token was kept"
    return "band"


def check_output(gpu_out: torch.Tensor, ref: np.ndarray, dtype, what=""):
    got = gpu_out.detach().float().cpu().numpy().reshape(ref.shape).astype(np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    tol = TOL[dtype]
    assert err.max() <= tol["max_abs"], f"{what}: max abs err {err.max():.3e} > {tol['max_abs']}"
    assert err.mean() <= tol["mean_abs"], f"{what}: mean abs err {err.mean():.3e} > {tol['mean_abs']}"
    return float(err.max()), float(err.mean())
