"""Python face of the fp64 CPU oracle (oracle/scalekv_oracle.c, oracle/selection_literal.c,
oracle/allocation.c).

TEST INFRASTRUCTURE.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this package.  It never imports the HIP binding and
the HIP binding never imports it.

All functions take numpy (or torch CPU) arrays of any float dtype, widen them
to float64 and call the C routines, one (sequence, head) unit per leading
index.  See the C file for what each step computes and which passage of the
paper it follows.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from .build import build as _build

_lib = None

_c_dp = ctypes.POINTER(ctypes.c_double)
_c_ip = ctypes.POINTER(ctypes.c_int32)


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build())
        _lib.scalekv_oracle_num_threads.restype = ctypes.c_int
        _lib.scalekv_oracle_cache_lengths.restype = ctypes.c_int
        _lib.scalekv_oracle_select.restype = ctypes.c_int
        _lib.scalekv_oracle_window_centroids.restype = ctypes.c_int
        _lib.scalekv_oracle_select_forced.restype = ctypes.c_int
        _lib.scalekv_oracle_step_append_first_batch.restype = ctypes.c_int
        _lib.scalekv_oracle_asi.restype = ctypes.c_double
        _lib.scalekv_oracle_drafters.restype = ctypes.c_int
        _lib.scalekv_oracle_budgets.restype = ctypes.c_int
        _lib.scalekv_oracle_positional.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().scalekv_oracle_num_threads())


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):  # torch tensor on the CPU
        x = x.detach().to("cpu").double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _dp(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_c_dp) if a is not None else None


def _ip(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_c_ip) if a is not None else None


def default_scale(d: int) -> float:
    return 1.0 / float(d) ** 0.5


def score(qw, k, scale: Optional[float] = None, return_attention: bool = False):
    """Eq. 5.  qw: [U, N, d] window queries, k: [U, len, d] cached keys.
    Returns (s [U, len], log_s [U, len]) and, if asked, the attention rows
    A [U, N, len]."""
    qw, k = _f64(qw), _f64(k)
    U, N, d = qw.shape
    L = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    s = np.zeros((U, L)); ls = np.zeros((U, L))
    a = np.zeros((U, N, L)) if return_attention else None
    for u in range(U):
        lib().scalekv_oracle_score(_dp(qw[u]), N, _dp(k[u]), L, d, ctypes.c_double(scale),
                                   _dp(s[u]), _dp(ls[u]), _dp(a[u]) if a is not None else None)
    return (s, ls, a) if return_attention else (s, ls)


def select(scores, budget: int) -> np.ndarray:
    """Top-min(budget, len) per unit, ties to the lower index, ascending.
    scores: [U, len] -> idx [U, keep] int32."""
    scores = _f64(scores)
    U, L = scores.shape
    keep = max(0, min(int(budget), L))
    idx = np.zeros((U, keep), dtype=np.int32)
    for u in range(U):
        got = lib().scalekv_oracle_select(_dp(scores[u]), L, int(budget), _ip(idx[u]))
        assert got == keep
    return idx


def compact(src, idx, cur) -> np.ndarray:
    """dst = [src[idx] ; cur] per unit.  src [U, len, d], idx [U, keep],
    cur [U, n_cur, d] -> [U, keep + n_cur, d] (float64 copies)."""
    src, cur = _f64(src), _f64(cur)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    U, _, d = src.shape
    keep, n_cur = idx.shape[1], cur.shape[1]
    dst = np.zeros((U, keep + n_cur, d))
    for u in range(U):
        lib().scalekv_oracle_compact(_dp(src[u]), _ip(idx[u]), keep, _dp(cur[u]), n_cur, d, _dp(dst[u]))
    return dst


def attend(q, k, v, scale: Optional[float] = None) -> np.ndarray:
    """Unmasked softmax attention per unit. q [U, n_q, d], k/v [U, kv, d]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    U, n_q, d = q.shape
    kv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    out = np.zeros((U, n_q, d))
    lib().scalekv_oracle_attend_batch(U, _dp(q), n_q, _dp(k), _dp(v), kv, d, ctypes.c_double(scale), _dp(out))
    return out


def step(q, k_cur, v_cur, win_idx: Sequence[int], k_src, v_src, budget: int,
         scale: Optional[float] = None, force_idx=None):
    """One (layer, scale) call: score -> select -> compact (+append) -> attend.
    q/k_cur/v_cur [U, n_cur, d]; k_src/v_src [U, cache_len, d].
    Returns dict(k_dst, v_dst [U, keep+n_cur, d], idx [U, keep], scores and
    log_scores [U, cache_len], out [U, n_cur, d], new_len).  The selection ranks
    on the log-scores."""
    q, k_cur, v_cur, k_src, v_src = map(_f64, (q, k_cur, v_cur, k_src, v_src))
    U, n_cur, d = q.shape
    L = k_src.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    win = np.ascontiguousarray(np.asarray(list(win_idx), dtype=np.int32))
    keep = max(0, min(int(budget), L))
    fidx = None
    if force_idx is not None:
        fidx = np.ascontiguousarray(np.asarray(force_idx, dtype=np.int32))
        keep = fidx.shape[1]
    k_dst = np.zeros((U, keep + n_cur, d)); v_dst = np.zeros((U, keep + n_cur, d))
    idx = np.zeros((U, keep), dtype=np.int32)
    sc = np.zeros((U, L)); lsc = np.zeros((U, L)); out = np.zeros((U, n_cur, d))
    lib().scalekv_oracle_step_batch(
        U, _dp(q), _dp(k_cur), _dp(v_cur), n_cur, _ip(win), len(win), _dp(k_src), _dp(v_src), L,
        int(budget), d, ctypes.c_double(scale), _ip(fidx), keep if fidx is not None else 0,
        _dp(k_dst), _dp(v_dst), _ip(idx), _dp(sc), _dp(lsc), _dp(out))
    return dict(k_dst=k_dst, v_dst=v_dst, idx=idx, scores=sc, log_scores=lsc, out=out, new_len=keep + n_cur)


def cache_lengths(prefix: int, n_tok: Sequence[int], budget: Sequence[int]) -> Tuple[np.ndarray, np.ndarray, int]:
    """(len entering each scale, keep at each scale, final length)."""
    n_tok = np.ascontiguousarray(np.asarray(n_tok, dtype=np.int32))
    budget = np.ascontiguousarray(np.asarray(budget, dtype=np.int32))
    K = len(n_tok)
    li = np.zeros(K, dtype=np.int32); kp = np.zeros(K, dtype=np.int32)
    final = lib().scalekv_oracle_cache_lengths(int(prefix), _ip(n_tok), _ip(budget), K, _ip(li), _ip(kp))
    return li, kp, int(final)


# ---- the literal reading of Sec. 3.3 (oracle/selection_literal.c)

def window_centroids(h: int, w: int, ph: int = 4, pw: int = 4) -> np.ndarray:
    """Raster indices of the centroid token of each patch of a ph x pw grid laid
    over an h x w token map (Sec. 3.3, observation window)."""
    idx = np.zeros(max(1, min(ph, h) * min(pw, w)), dtype=np.int32)
    n = lib().scalekv_oracle_window_centroids(int(h), int(w), int(ph), int(pw), _ip(idx))
    return idx[:n].copy()


def pool(scores, pool_w: int) -> np.ndarray:
    """Average pooling along the cache axis, odd width, zero padding. [U, len] -> [U, len]."""
    scores = _f64(scores)
    out = np.zeros_like(scores)
    for u in range(scores.shape[0]):
        lib().scalekv_oracle_pool(_dp(scores[u]), scores.shape[1], int(pool_w), _dp(out[u]))
    return out


def pool_log(log_scores, pool_w: int) -> np.ndarray:
    """The same pooling on log-scores: log of the average of exp(log_scores) over the window,
    finite where the scores themselves underflow. [U, len] -> [U, len]."""
    ls = _f64(log_scores)
    out = np.zeros_like(ls)
    for u in range(ls.shape[0]):
        lib().scalekv_oracle_pool_log(_dp(ls[u]), ls.shape[1], int(pool_w), _dp(out[u]))
    return out


def select_forced(scores, budget: int, forced: Sequence[int]) -> np.ndarray:
    """Forced positions plus the top-min(budget, rest) of the others, ascending.
    scores [U, len] -> idx [U, keep]."""
    scores = _f64(scores)
    U, L = scores.shape
    f = np.ascontiguousarray(np.asarray(list(forced), dtype=np.int32))
    buf = np.zeros((U, max(L, 1)), dtype=np.int32)
    keep = None
    for u in range(U):
        got = lib().scalekv_oracle_select_forced(_dp(scores[u]), L, int(budget), _ip(f), len(f), _ip(buf[u]))
        assert keep is None or got == keep
        keep = got
    return buf[:, :keep or 0].copy()


def step_append_first(q, k_cur, v_cur, win_idx: Sequence[int], k_cache, v_cache, budget: int,
                      pool_w: int = 1, scale: Optional[float] = None, force_idx=None):
    """One (layer, scale) call in the order of Sec. 3.3: append -> attend ->
    score over history and current map -> pool -> keep window + top-budget.
    Returns dict(out [U, n_cur, d], scores and log_scores [U, len] (pooled), idx [U, keep],
    k_next, v_next [U, keep, d], keep) with len = cache_len + n_cur."""
    q, k_cur, v_cur, k_cache, v_cache = map(_f64, (q, k_cur, v_cur, k_cache, v_cache))
    U, n_cur, d = q.shape
    L = k_cache.shape[1]
    n = L + n_cur
    scale = default_scale(d) if scale is None else float(scale)
    win = np.ascontiguousarray(np.asarray(list(win_idx), dtype=np.int32))
    fidx, fkeep = None, 0
    if force_idx is not None:
        fidx = np.ascontiguousarray(np.asarray(force_idx, dtype=np.int32))
        fkeep = fidx.shape[1]
    k_next = np.zeros((U, n, d)); v_next = np.zeros((U, n, d))
    idx = np.zeros((U, n), dtype=np.int32)
    sc = np.zeros((U, n)); lsc = np.zeros((U, n)); out = np.zeros((U, n_cur, d))
    keep = lib().scalekv_oracle_step_append_first_batch(
        U, _dp(q), _dp(k_cur), _dp(v_cur), n_cur, _ip(win), len(win), int(pool_w), _dp(k_cache),
        _dp(v_cache), L, int(budget), d, ctypes.c_double(scale), _ip(fidx), fkeep, _dp(k_next),
        _dp(v_next), _ip(idx), _dp(sc), _dp(lsc), _dp(out))
    return dict(out=out, scores=sc, log_scores=lsc, idx=idx[:, :keep].copy(), k_next=k_next[:, :keep].copy(),
                v_next=v_next[:, :keep].copy(), keep=int(keep))


# ---- the offline policy: ASI, drafter set, budgets, comparison policies (oracle/allocation.c)

def asi_terms(q, k, hist_len: int, top_k: int, scale: Optional[float] = None):
    """Eq. 2, both factors per sampled query.  q [U, n_s, d]; k [U, hist_len + cur_len, d]
    (history rows first).  Returns (cur_ratio [U, n_s], hist_topk [U, n_s])."""
    q, k = _f64(q), _f64(k)
    U, n_s, d = q.shape
    cur_len = k.shape[1] - int(hist_len)
    scale = default_scale(d) if scale is None else float(scale)
    cur = np.zeros((U, n_s)); top = np.zeros((U, n_s))
    for u in range(U):
        lib().scalekv_oracle_asi_terms(_dp(q[u]), n_s, _dp(k[u]), int(hist_len), cur_len, d,
                                       ctypes.c_double(scale), int(top_k), _dp(cur[u]), _dp(top[u]))
    return cur, top


def asi(cur_ratio, hist_topk) -> float:
    """Eq. 2: product of the two means over every sampled query handed in."""
    a, b = _f64(cur_ratio).ravel(), _f64(hist_topk).ravel()
    return float(lib().scalekv_oracle_asi(_dp(a), _dp(b), a.size))


def zscores(asi_lk, eps: float = 1e-8) -> np.ndarray:
    """Eq. 3: per-scale Z-score of ASI [L, K]."""
    a = _f64(asi_lk)
    L, K = a.shape
    z = np.zeros((L, K))
    lib().scalekv_oracle_zscores(_dp(a), L, K, ctypes.c_double(eps), _dp(z))
    return z


def drafters(z, n_d: int) -> np.ndarray:
    """Eq. 3: [L, K] int32 mask of the n_d pairs with the lowest Z."""
    z = _f64(z)
    L, K = z.shape
    mask = np.zeros((L, K), dtype=np.int32)
    lib().scalekv_oracle_drafters(_dp(z), L, K, int(n_d), _ip(mask))
    return mask


def budgets(L: int, n_d: Sequence[int], b_uniform: int, b_r0: int, delta: int, b_min: int = 0):
    """Eq. 4 -> (b_r [K], b_d, slack) or None when it has no solution."""
    n_d = np.ascontiguousarray(np.asarray(list(n_d), dtype=np.int32))
    K = len(n_d)
    b_r = np.zeros(K, dtype=np.int32)
    b_d = ctypes.c_int32(0); slack = ctypes.c_longlong(0)
    rc = lib().scalekv_oracle_budgets(int(L), K, _ip(n_d), ctypes.c_longlong(b_uniform),
                                      ctypes.c_longlong(b_r0), ctypes.c_longlong(delta),
                                      ctypes.c_longlong(b_min), _ip(b_r), ctypes.byref(b_d),
                                      ctypes.byref(slack))
    if rc != 0:
        return None
    return b_r, int(b_d.value), int(slack.value)


def positional(length: int, n_sink: int, n_recent: int) -> np.ndarray:
    """Sliding-window / sinks-and-recent positions of Sec. 4.1, ascending."""
    idx = np.zeros(max(1, length), dtype=np.int32)
    n = lib().scalekv_oracle_positional(int(length), int(n_sink), int(n_recent), _ip(idx))
    return idx[:n].copy()


def pyramid(L: int, b_uniform: int, b_last: int) -> np.ndarray:
    """Pyramid-shaped per-layer budgets of Sec. 4.1 with mean b_uniform."""
    b = np.zeros(L, dtype=np.int32)
    lib().scalekv_oracle_pyramid(int(L), ctypes.c_longlong(b_uniform), ctypes.c_longlong(b_last), _ip(b))
    return b
