"""Shared helpers for the GPU parity tests: the comparison rules only.
(No method arithmetic: expected values always come from `oracle`.)"""
from __future__ import annotations

import numpy as np
import torch

REL_MARGIN = 1e-4          # k-th / (k+1)-th score margin above which indices must match exactly
TOL = {torch.float32: dict(max_abs=1e-4, mean_abs=1e-4),
       torch.bfloat16: dict(max_abs=2e-2, mean_abs=1e-2)}
# A bf16 output cannot be closer to the exact value than its own rounding allows: half an ulp is
# 2^-8 of the value at the bottom of a binade (3.1e-2 for an output of 8), and the probabilities
# that multiply V carry 2^-9 of their own.  So an element of magnitude above 2.56 (= 2e-2 * 2^7)
# is held to 2^-7 of its magnitude instead of to 2e-2; below that the absolute bound rules.
BF16_REL = 2.0 ** -7


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
    lim = np.full_like(err, tol["max_abs"])
    if dtype == torch.bfloat16:
        lim = np.maximum(lim, BF16_REL * np.abs(ref))
    worst = np.unravel_index(np.argmax(err - lim), err.shape)
    assert np.all(err <= lim), (f"{what}: abs err {err[worst]:.3e} > {lim[worst]:.3e} "
                                f"at an output of {ref[worst]:.3f}")
    assert err.mean() <= tol["mean_abs"], f"{what}: mean abs err {err.mean():.3e} > {tol['mean_abs']}"
    return float(err.max()), float(err.mean())
