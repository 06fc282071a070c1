"""Shared helpers for the GPU parity tests: the comparison rules only.
(No method arithmetic: expected values always come from `oracle`.)"""
from __future__ import annotations

import numpy as np
import torch

REL_MARGIN = 1e-4          # k-th / (k+1)-th score margin above which indices must match exactly
TOL = {torch.float32: dict(max_abs=1e-4, mean_abs=1e-4),
       torch.bfloat16: dict(max_abs=2e-2, mean_abs=1e-2)}
# bf16 outputs: 2e-2 absolute for every element whose exact value is below 8 in magnitude.  From 8
# up no bf16 number can promise that (half an ulp of a value in [8, 16) is 3.1e-2), so such an
# element is held to what the arithmetic carries: half a bf16 ulp of the exact value's binade (the
# output rounding) plus 2^-9 of its magnitude (the probabilities are rounded to bf16, 2^-9 relative,
# before they multiply V).  At 8 that is 4.7e-2.
BF16_ABS_BELOW = 8.0
BF16_P_REL = 2.0 ** -9
STATS = dict(bf16_elements=0, bf16_wide=0, bf16_wide_max_err=0.0, bf16_max_err_below_8=0.0)


def bf16_half_ulp(x: np.ndarray) -> np.ndarray:
    """half the spacing of bf16 numbers (8 significant bits) in the binade of |x| (x != 0)"""
    _, e = np.frexp(np.abs(x))              # |x| = m * 2^e, m in [0.5, 1)
    return np.ldexp(1.0, e - 1 - 7 - 1)     # ulp = 2^(e-1-7)


def units(t: torch.Tensor) -> torch.Tensor:
    """[S,H,rows,d] -> [S*H,rows,d] on the CPU."""
    return t.detach().cpu().reshape(t.shape[0] * t.shape[1], *t.shape[2:])


def check_indices(gpu_idx: np.ndarray, log_scores: np.ndarray, keep: int, oracle_idx: np.ndarray):
    """Index rule for one unit.  log_scores: the oracle's fp64 log-scores (finite).
    The rule is the one on the scores themselves, written on their logarithms so that it also
    holds where the scores underflow: with a, b the keep-th and (keep+1)-th largest scores,
    (a - b) / a > REL_MARGIN  <=>  log b - log a < log(1 - REL_MARGIN)  -> the GPU list must equal
    the oracle's; otherwise it must be a valid choice inside the near-tie band, i.e. contain every
    token with s > a (1 + REL_MARGIN) and none with s < a (1 - REL_MARGIN).
    Returns 'exact' or 'band'."""
    gpu_idx = np.asarray(gpu_idx)
    ls = np.asarray(log_scores, dtype=np.float64)
    n = len(ls)
    assert gpu_idx.shape == (keep,)
    assert np.all(np.diff(gpu_idx) > 0), "indices must be strictly ascending (no duplicates)"
    if keep:
        assert gpu_idx[0] >= 0 and gpu_idx[-1] < n
    if keep == 0 or keep == n:
        assert np.array_equal(gpu_idx, oracle_idx)
        return "exact"
    order = np.sort(ls)[::-1]
    la, lb = order[keep - 1], order[keep]
    assert np.isfinite(la), "the keep-th log-score is not finite: the rule would accept anything"
    if lb - la < np.log1p(-REL_MARGIN):
        assert np.array_equal(gpu_idx, oracle_idx), "indices differ although the margin is wide"
        return "exact"
    chosen = np.zeros(n, dtype=bool); chosen[gpu_idx] = True
    must = ls > la + np.log1p(REL_MARGIN)
    may = ls >= la + np.log1p(-REL_MARGIN)
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
        wide = np.abs(ref) >= BF16_ABS_BELOW
        STATS["bf16_elements"] += err.size
        if wide.any():
            lim[wide] = bf16_half_ulp(ref[wide]) + BF16_P_REL * np.abs(ref[wide])
            STATS["bf16_wide"] += int(wide.sum())
            STATS["bf16_wide_max_err"] = max(STATS["bf16_wide_max_err"], float(err[wide].max()))
            print(f"  {what}: {int(wide.sum())} of {err.size} outputs at or above {BF16_ABS_BELOW:g} in magnitude "
                  f"(largest error among them {err[wide].max():.3e}, limit there {lim[wide].min():.3e} and up)", flush=True)
        if (~wide).any():
            STATS["bf16_max_err_below_8"] = max(STATS["bf16_max_err_below_8"], float(err[~wide].max()))
    worst = np.unravel_index(np.argmax(err - lim), err.shape)
    assert np.all(err <= lim), (f"{what}: abs err {err[worst]:.3e} > {lim[worst]:.3e} "
                                f"at an output of {ref[worst]:.3f}")
    assert err.mean() <= tol["mean_abs"], f"{what}: mean abs err {err.mean():.3e} > {tol['mean_abs']}"
    return float(err.max()), float(err.mean())
