"""ctypes binding with the same names as the C entry points.

Each function checks tensor dtype/device/contiguity (so that a pointer handed
to C means what the header says), passes raw device pointers, sizes and the
current HIP stream, and raises ScaleKVError on a non-OK status.  No arithmetic
happens here.  Where a tensor's shape depends on how many rows a call keeps
(idx [S,H,keep]), the binding works the number out only to check that shape
before the call; what it returns is always the value the library wrote, and
the two are asserted equal.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
MAX_WINDOW = 16

MAX_POOL = 31
MAX_ASI_SAMPLES = 1024
STATIC_SCRATCH_BYTES = 64 << 20   # SCALEKV_STATIC_SCRATCH_BYTES

# status-returning entry points first, then the two that return strings
_STATUS_SYMBOLS = (
    "scalekv_workspace_bytes", "scalekv_score", "scalekv_select", "scalekv_compact",
    "scalekv_attend", "scalekv_step", "scalekv_step_static", "scalekv_step_stage_events",
    "scalekv_window_centroids", "scalekv_select_window", "scalekv_step_append_first",
    "scalekv_asi", "scalekv_drafter_set", "scalekv_allocate_budgets", "scalekv_select_positional",
    "scalekv_pyramid_budgets", "scalekv_policy_table",
)
EXPORTED_SYMBOLS = _STATUS_SYMBOLS + ("scalekv_last_error", "scalekv_version")

_STATUS = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE", 4: "HIP"}


class ScaleKVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"scalekv status {status} ({_STATUS.get(status, '?')}): {message}")
        self.status = status


class _CShape(ctypes.Structure):
    _fields_ = [("n_seq", ctypes.c_int32), ("n_head", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float)]


class _CKv(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("seq_stride", ctypes.c_int64),
                ("head_stride", ctypes.c_int64), ("capacity", ctypes.c_int32)]


_DTYPES = {torch.float32: 0, torch.bfloat16: 1}


@dataclass(frozen=True)
class Shape:
    n_seq: int
    n_head: int
    head_dim: int
    dtype: torch.dtype
    sm_scale: float = 0.0   # <= 0: 1/sqrt(head_dim)

    def c(self) -> _CShape:
        if self.dtype not in _DTYPES:
            raise ScaleKVError(2, f"dtype {self.dtype} is not float32 or bfloat16")
        return _CShape(self.n_seq, self.n_head, self.head_dim, _DTYPES[self.dtype], float(self.sm_scale))


_lib: Optional[ctypes.CDLL] = None


def lib_path() -> str:
    """The library built in-tree.  SCALEKV_LIBRARY (a path) overrides it: a measurement aid for
    the ablation builds of `build.py --variant`, whose results are wrong on purpose."""
    return os.environ.get("SCALEKV_LIBRARY") or os.path.join(HERE, "libscalekv.so")


def lib() -> ctypes.CDLL:
    """Load libscalekv.so (built in-tree by paper_2505_19602_amd/build.py)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2505_19602_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(path)
        L.scalekv_last_error.restype = ctypes.c_char_p
        L.scalekv_version.restype = ctypes.c_char_p
        for name in _STATUS_SYMBOLS:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def version() -> str:
    return lib().scalekv_version().decode()


def _check(status: int) -> None:
    if status != 0:
        raise ScaleKVError(status, lib().scalekv_last_error().decode())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _dense(t: torch.Tensor, shape: Shape, rows: int, name: str, dtype=None) -> torch.Tensor:
    want = (shape.n_seq, shape.n_head, rows, shape.head_dim)
    if tuple(t.shape) != want:
        raise ScaleKVError(1, f"{name} has shape {tuple(t.shape)}, expected {want}")
    if t.dtype != (dtype or shape.dtype):
        raise ScaleKVError(1, f"{name} has dtype {t.dtype}, expected {dtype or shape.dtype}")
    if not t.is_cuda or not t.is_contiguous():
        raise ScaleKVError(1, f"{name} must be a contiguous device tensor")
    return t


def _kv(t: torch.Tensor, shape: Shape, name: str) -> _CKv:
    """[S,H,capacity,d] tensor (a view with larger strides is fine as long as
    rows are contiguous) -> scalekv_kv."""
    if t.dim() != 4 or t.shape[0] != shape.n_seq or t.shape[1] != shape.n_head or t.shape[3] != shape.head_dim:
        raise ScaleKVError(1, f"{name} has shape {tuple(t.shape)}, expected [S,H,capacity,d]")
    if t.dtype != shape.dtype or not t.is_cuda:
        raise ScaleKVError(1, f"{name} must be a device tensor of dtype {shape.dtype}")
    if t.stride(3) != 1 or t.stride(2) != shape.head_dim:
        raise ScaleKVError(1, f"{name}: rows must be contiguous (strides {t.stride()})")
    return _CKv(t.data_ptr(), t.stride(0), t.stride(1), t.shape[2])


def workspace_bytes(shape: Shape, max_cache_len: int, max_q: int) -> int:
    out = ctypes.c_size_t(0)
    cs = shape.c()
    _check(lib().scalekv_workspace_bytes(ctypes.byref(cs), int(max_cache_len), int(max_q), ctypes.byref(out)))
    return int(out.value)


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return ctypes.c_void_p(0), ctypes.c_size_t(0)
    if not ws.is_cuda or not ws.is_contiguous():
        raise ScaleKVError(1, "workspace must be a contiguous device tensor")
    return ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel() * ws.element_size())


def score(shape: Shape, q_win: torch.Tensor, k: torch.Tensor, cache_len: int,
          log_scores: torch.Tensor, ws: torch.Tensor) -> None:
    """scalekv_score: q_win [S,H,n_win,d], k cache [S,H,cap,d] -> log_scores [S,H,cache_len] fp32."""
    n_win = q_win.shape[2]
    _dense(q_win, shape, n_win, "q_win")
    if tuple(log_scores.shape) != (shape.n_seq, shape.n_head, cache_len) or log_scores.dtype != torch.float32 \
            or not log_scores.is_cuda or not log_scores.is_contiguous():
        raise ScaleKVError(1, "log_scores must be a contiguous fp32 device tensor [S,H,cache_len]")
    cs, ck = shape.c(), _kv(k, shape, "k")
    wp, wb = _ws(ws)
    _check(lib().scalekv_score(ctypes.byref(cs), _ptr(q_win), int(n_win), ctypes.byref(ck), int(cache_len),
                               _ptr(log_scores), wp, wb, _stream()))


def select(shape: Shape, scores: torch.Tensor, cache_len: int, budget: int, idx: torch.Tensor) -> int:
    """scalekv_select: scores [S,H,cache_len] fp32 -> idx [S,H,keep] int32; returns keep."""
    if scores.dtype != torch.float32 or not scores.is_cuda or not scores.is_contiguous() \
            or tuple(scores.shape) != (shape.n_seq, shape.n_head, cache_len):
        raise ScaleKVError(1, "scores must be a contiguous fp32 device tensor [S,H,cache_len]")
    keep = max(0, min(int(budget), int(cache_len)))
    if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous() \
            or tuple(idx.shape) != (shape.n_seq, shape.n_head, keep):
        raise ScaleKVError(1, f"idx must be a contiguous int32 device tensor [S,H,{keep}]")
    cs = shape.c()
    out = ctypes.c_int32(-1)
    _check(lib().scalekv_select(ctypes.byref(cs), _ptr(scores), int(cache_len), int(budget), _ptr(idx),
                                ctypes.byref(out), _stream()))
    assert out.value == keep, "the binding's shape check and the library disagree on keep"
    return int(out.value)


def compact(shape: Shape, k_src: torch.Tensor, v_src: torch.Tensor, cache_len: int,
            idx: Optional[torch.Tensor], keep: int, k_cur: Optional[torch.Tensor],
            v_cur: Optional[torch.Tensor], k_dst: torch.Tensor, v_dst: torch.Tensor) -> int:
    """scalekv_compact; returns keep + n_cur."""
    n_cur = 0 if k_cur is None else k_cur.shape[2]
    if k_cur is not None:
        _dense(k_cur, shape, n_cur, "k_cur")
        _dense(v_cur, shape, n_cur, "v_cur")
    if idx is not None:
        if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous() \
                or tuple(idx.shape) != (shape.n_seq, shape.n_head, keep):
            raise ScaleKVError(1, f"idx must be a contiguous int32 device tensor [S,H,{keep}]")
    cs = shape.c()
    a, b, c, d = _kv(k_src, shape, "k_src"), _kv(v_src, shape, "v_src"), _kv(k_dst, shape, "k_dst"), _kv(v_dst, shape, "v_dst")
    _check(lib().scalekv_compact(ctypes.byref(cs), ctypes.byref(a), ctypes.byref(b), int(cache_len), _ptr(idx),
                                 int(keep), _ptr(k_cur), _ptr(v_cur), int(n_cur), ctypes.byref(c),
                                 ctypes.byref(d), _stream()))
    return keep + n_cur


def attend(shape: Shape, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, kv_len: int,
           out: torch.Tensor) -> None:
    """scalekv_attend: q [S,H,n_q,d], caches k/v (first kv_len rows) -> out [S,H,n_q,d]."""
    n_q = q.shape[2]
    _dense(q, shape, n_q, "q")
    _dense(out, shape, n_q, "out")
    cs, ck, cv = shape.c(), _kv(k, shape, "k"), _kv(v, shape, "v")
    _check(lib().scalekv_attend(ctypes.byref(cs), _ptr(q), int(n_q), ctypes.byref(ck), ctypes.byref(cv),
                                int(kv_len), _ptr(out), _stream()))


def step(shape: Shape, q: torch.Tensor, k_cur: torch.Tensor, v_cur: torch.Tensor,
         win_idx: Sequence[int], k_src: torch.Tensor, v_src: torch.Tensor, cache_len: int, budget: int,
         k_dst: torch.Tensor, v_dst: torch.Tensor, out: torch.Tensor,
         idx_out: Optional[torch.Tensor], ws: Optional[torch.Tensor]) -> int:
    """scalekv_step; returns the new cache length keep + n_cur."""
    n_cur = q.shape[2]
    _dense(q, shape, n_cur, "q"); _dense(k_cur, shape, n_cur, "k_cur"); _dense(v_cur, shape, n_cur, "v_cur")
    _dense(out, shape, n_cur, "out")
    keep = max(0, min(int(budget), int(cache_len)))
    if idx_out is not None:
        if idx_out.dtype != torch.int32 or not idx_out.is_cuda or not idx_out.is_contiguous() \
                or tuple(idx_out.shape) != (shape.n_seq, shape.n_head, keep):
            raise ScaleKVError(1, f"idx_out must be a contiguous int32 device tensor [S,H,{keep}]")
    win = (ctypes.c_int32 * max(1, len(win_idx)))(*[int(w) for w in win_idx])
    cs = shape.c()
    a, b, c, d = _kv(k_src, shape, "k_src"), _kv(v_src, shape, "v_src"), _kv(k_dst, shape, "k_dst"), _kv(v_dst, shape, "v_dst")
    wp, wb = _ws(ws)
    new_len = ctypes.c_int32(-1)
    _check(lib().scalekv_step(ctypes.byref(cs), _ptr(q), _ptr(k_cur), _ptr(v_cur), int(n_cur), win,
                              int(len(win_idx)), ctypes.byref(a), ctypes.byref(b), int(cache_len), int(budget),
                              ctypes.byref(c), ctypes.byref(d), ctypes.byref(new_len), _ptr(out), _ptr(idx_out),
                              wp, wb, _stream()))
    assert new_len.value == keep + n_cur, "the binding's shape check and the library disagree on keep"
    return int(new_len.value)


def step_static(shape: Shape, q: torch.Tensor, k_cur: torch.Tensor, v_cur: torch.Tensor,
                win_idx: Sequence[int], k_src: torch.Tensor, v_src: torch.Tensor, cache_len: int, budget: int,
                k_dst: torch.Tensor, v_dst: torch.Tensor, out: torch.Tensor,
                idx_out: Optional[torch.Tensor]) -> int:
    """scalekv_step_static: the step with the library's own fixed scratch array instead of a
    caller workspace (allocates nothing); returns the new cache length."""
    n_cur = q.shape[2]
    _dense(q, shape, n_cur, "q"); _dense(k_cur, shape, n_cur, "k_cur"); _dense(v_cur, shape, n_cur, "v_cur")
    _dense(out, shape, n_cur, "out")
    if idx_out is not None and (idx_out.dtype != torch.int32 or not idx_out.is_cuda or not idx_out.is_contiguous()
                                or idx_out.dim() != 3 or tuple(idx_out.shape[:2]) != (shape.n_seq, shape.n_head)):
        raise ScaleKVError(1, "idx_out must be a contiguous int32 device tensor [S,H,keep]")
    win = (ctypes.c_int32 * max(1, len(win_idx)))(*[int(w) for w in win_idx])
    cs = shape.c()
    a, b, c, d = _kv(k_src, shape, "k_src"), _kv(v_src, shape, "v_src"), _kv(k_dst, shape, "k_dst"), _kv(v_dst, shape, "v_dst")
    new_len = ctypes.c_int32(-1)
    _check(lib().scalekv_step_static(ctypes.byref(cs), _ptr(q), _ptr(k_cur), _ptr(v_cur), int(n_cur), win,
                                     int(len(win_idx)), ctypes.byref(a), ctypes.byref(b), int(cache_len),
                                     int(budget), ctypes.byref(c), ctypes.byref(d), ctypes.byref(new_len),
                                     _ptr(out), _ptr(idx_out), _stream()))
    if idx_out is not None and idx_out.shape[2] != new_len.value - n_cur:
        raise ScaleKVError(1, f"idx_out holds {idx_out.shape[2]} entries per unit, the step kept {new_len.value - n_cur}")
    return int(new_len.value)


class PreparedStep:
    """One scalekv_step call with every argument already marshalled.  Building it does
    all the checks that `step` does; calling it only crosses into C, which matters for
    the small scales where a call's own work is a few microseconds.  Holds references to
    its tensors so the pointers stay valid."""

    __slots__ = ("_args", "_keep", "new_len", "_refs", "_fn")

    def __init__(self, shape: Shape, q, k_cur, v_cur, win_idx, k_src, v_src, cache_len, budget,
                 k_dst, v_dst, out, idx_out, ws):
        n_cur = q.shape[2]
        _dense(q, shape, n_cur, "q"); _dense(k_cur, shape, n_cur, "k_cur"); _dense(v_cur, shape, n_cur, "v_cur")
        _dense(out, shape, n_cur, "out")
        keep = max(0, min(int(budget), int(cache_len)))
        if idx_out is not None:
            if idx_out.dtype != torch.int32 or not idx_out.is_cuda or not idx_out.is_contiguous() \
                    or tuple(idx_out.shape) != (shape.n_seq, shape.n_head, keep):
                raise ScaleKVError(1, f"idx_out must be a contiguous int32 device tensor [S,H,{keep}]")
        win = (ctypes.c_int32 * max(1, len(win_idx)))(*[int(w) for w in win_idx])
        cs = shape.c()
        a, b = _kv(k_src, shape, "k_src"), _kv(v_src, shape, "v_src")
        c, d = _kv(k_dst, shape, "k_dst"), _kv(v_dst, shape, "v_dst")
        wp, wb = _ws(ws)
        new_len = ctypes.c_int32(-1)
        self._refs = (cs, win, a, b, c, d, new_len, q, k_cur, v_cur, k_src, v_src, k_dst, v_dst, out, idx_out, ws)
        self._args = [ctypes.byref(cs), _ptr(q), _ptr(k_cur), _ptr(v_cur), ctypes.c_int32(n_cur), win,
                      ctypes.c_int32(len(win_idx)), ctypes.byref(a), ctypes.byref(b), ctypes.c_int32(cache_len),
                      ctypes.c_int32(budget), ctypes.byref(c), ctypes.byref(d), ctypes.byref(new_len), _ptr(out),
                      _ptr(idx_out), wp, wb, None]
        self._keep = keep
        self.new_len = keep + n_cur
        self._fn = lib().scalekv_step

    def __call__(self, stream_ptr: Optional[int] = None) -> int:
        """Enqueue on `stream_ptr` (a hipStream_t as int) or on torch's current stream."""
        args = self._args
        args[-1] = ctypes.c_void_p(stream_ptr if stream_ptr is not None
                                   else torch.cuda.current_stream().cuda_stream)
        status = self._fn(*args)
        if status != 0:
            _check(status)
        assert self._refs[6].value == self.new_len, "the binding's shape check and the library disagree on keep"
        return self.new_len


class PreparedAppendFirst:
    """One scalekv_step_append_first call with every argument already marshalled (see
    PreparedStep).  `keep` and `moved` are known on the host before anything runs."""

    __slots__ = ("_args", "keep", "moved", "_refs", "_fn")

    def __init__(self, shape: Shape, q, k_cur, v_cur, win_idx, pool_w, k_cache, v_cache, cache_len, budget,
                 k_next, v_next, out, idx_out, ws):
        n_cur = q.shape[2]
        _dense(q, shape, n_cur, "q"); _dense(k_cur, shape, n_cur, "k_cur"); _dense(v_cur, shape, n_cur, "v_cur")
        _dense(out, shape, n_cur, "out")
        total = int(cache_len) + n_cur
        self.keep = len(win_idx) + max(0, min(int(budget), total - len(win_idx)))
        self.moved = self.keep < total
        _idx_tensor(idx_out, shape, self.keep, "idx_out")
        win = (ctypes.c_int32 * max(1, len(win_idx)))(*[int(w) for w in win_idx])
        cs = shape.c()
        a, b = _kv(k_cache, shape, "k_cache"), _kv(v_cache, shape, "v_cache")
        c = _kv(k_next, shape, "k_next") if k_next is not None else None
        d = _kv(v_next, shape, "v_next") if v_next is not None else None
        wp, wb = _ws(ws)
        keep_out, moved = ctypes.c_int32(-1), ctypes.c_int32(-1)
        self._refs = (cs, win, a, b, c, d, keep_out, moved, q, k_cur, v_cur, k_cache, v_cache, k_next, v_next, out,
                      idx_out, ws)
        self._args = [ctypes.byref(cs), _ptr(q), _ptr(k_cur), _ptr(v_cur), ctypes.c_int32(n_cur), win,
                      ctypes.c_int32(len(win_idx)), ctypes.c_int32(pool_w), ctypes.byref(a), ctypes.byref(b),
                      ctypes.c_int32(cache_len), ctypes.c_int32(budget),
                      ctypes.byref(c) if c is not None else None, ctypes.byref(d) if d is not None else None,
                      ctypes.byref(keep_out), ctypes.byref(moved), _ptr(out), _ptr(idx_out), wp, wb, None]
        self._fn = lib().scalekv_step_append_first

    def __call__(self, stream_ptr: Optional[int] = None) -> int:
        args = self._args
        args[-1] = ctypes.c_void_p(stream_ptr if stream_ptr is not None
                                   else torch.cuda.current_stream().cuda_stream)
        status = self._fn(*args)
        if status != 0:
            _check(status)
        assert self._refs[6].value == self.keep and bool(self._refs[7].value) == self.moved, \
            "the binding's shape check and the library disagree on keep / moved"
        return self.keep


def step_stage_events(events) -> None:
    """scalekv_step_stage_events: `events` is a ctypes array of 5 hipEvent_t
    (c_void_p) or None."""
    _check(lib().scalekv_step_stage_events(events))


# ---- Sec. 3.3 read literally: append, attend, then prune with the window preserved

def window_centroids(map_h: int, map_w: int, patch_rows: int = 4, patch_cols: int = 4) -> list:
    """scalekv_window_centroids: raster indices of the centroid token of each patch."""
    cap = max(1, min(int(patch_rows), int(map_h)) * min(int(patch_cols), int(map_w)))
    buf = (ctypes.c_int32 * cap)()
    n = ctypes.c_int32(0)
    _check(lib().scalekv_window_centroids(int(map_h), int(map_w), int(patch_rows), int(patch_cols), buf,
                                          ctypes.byref(n)))
    return [int(buf[i]) for i in range(n.value)]


def _idx_tensor(t: Optional[torch.Tensor], shape: Shape, keep: int, name: str) -> None:
    if t is None:
        return
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() \
            or tuple(t.shape) != (shape.n_seq, shape.n_head, keep):
        raise ScaleKVError(1, f"{name} must be a contiguous int32 device tensor [S,H,{keep}]")


def select_window(shape: Shape, log_scores: torch.Tensor, cache_len: int, budget: int,
                  forced: Sequence[int], pool_w: int, idx: torch.Tensor) -> int:
    """scalekv_select_window: forced positions + top-budget of the rest by pooled score; returns keep."""
    if log_scores.dtype != torch.float32 or not log_scores.is_cuda or not log_scores.is_contiguous() \
            or tuple(log_scores.shape) != (shape.n_seq, shape.n_head, cache_len):
        raise ScaleKVError(1, "log_scores must be a contiguous fp32 device tensor [S,H,cache_len]")
    keep = len(forced) + max(0, min(int(budget), int(cache_len) - len(forced)))
    _idx_tensor(idx, shape, keep, "idx")
    f = (ctypes.c_int32 * max(1, len(forced)))(*[int(x) for x in forced])
    cs = shape.c()
    out = ctypes.c_int32(-1)
    _check(lib().scalekv_select_window(ctypes.byref(cs), _ptr(log_scores), int(cache_len), int(budget), f,
                                       int(len(forced)), int(pool_w), _ptr(idx), ctypes.byref(out), _stream()))
    assert out.value == keep, "the binding's shape check and the library disagree on keep"
    return int(out.value)


def step_append_first(shape: Shape, q: torch.Tensor, k_cur: torch.Tensor, v_cur: torch.Tensor,
                      win_idx: Sequence[int], pool_w: int, k_cache: torch.Tensor, v_cache: torch.Tensor,
                      cache_len: int, budget: int, k_next: Optional[torch.Tensor],
                      v_next: Optional[torch.Tensor], out: torch.Tensor, idx_out: Optional[torch.Tensor],
                      ws: Optional[torch.Tensor]):
    """scalekv_step_append_first; returns (keep, moved): the next cache has `keep` rows and
    lives in k_next/v_next if `moved`, else still in k_cache/v_cache."""
    n_cur = q.shape[2]
    _dense(q, shape, n_cur, "q"); _dense(k_cur, shape, n_cur, "k_cur"); _dense(v_cur, shape, n_cur, "v_cur")
    _dense(out, shape, n_cur, "out")
    total = int(cache_len) + n_cur
    keep = len(win_idx) + max(0, min(int(budget), total - len(win_idx)))
    _idx_tensor(idx_out, shape, keep, "idx_out")
    win = (ctypes.c_int32 * max(1, len(win_idx)))(*[int(w) for w in win_idx])
    cs = shape.c()
    a, b = _kv(k_cache, shape, "k_cache"), _kv(v_cache, shape, "v_cache")
    c = _kv(k_next, shape, "k_next") if k_next is not None else None
    d = _kv(v_next, shape, "v_next") if v_next is not None else None
    wp, wb = _ws(ws)
    keep_out, moved = ctypes.c_int32(-1), ctypes.c_int32(-1)
    _check(lib().scalekv_step_append_first(
        ctypes.byref(cs), _ptr(q), _ptr(k_cur), _ptr(v_cur), int(n_cur), win, int(len(win_idx)), int(pool_w),
        ctypes.byref(a), ctypes.byref(b), int(cache_len), int(budget),
        ctypes.byref(c) if c is not None else None, ctypes.byref(d) if d is not None else None,
        ctypes.byref(keep_out), ctypes.byref(moved), _ptr(out), _ptr(idx_out), wp, wb, _stream()))
    assert keep_out.value == keep, "the binding's shape check and the library disagree on keep"
    return int(keep_out.value), bool(moved.value)


# ---- the offline policy (Eq. 2-4) and the comparison policies of Sec. 4.1

def asi(shape: Shape, q_samp: torch.Tensor, k: torch.Tensor, hist_len: int, cur_len: int, top_k: int,
        terms: torch.Tensor, asi_out: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    """scalekv_asi: q_samp [S,H,n_samp,d], k cache (history rows then the current map) ->
    terms [S,H,n_samp,2] fp32 and, if given, asi_out [3] fp32 (two means and their product)."""
    n_samp = q_samp.shape[2]
    _dense(q_samp, shape, n_samp, "q_samp")
    if terms.dtype != torch.float32 or not terms.is_cuda or not terms.is_contiguous() \
            or tuple(terms.shape) != (shape.n_seq, shape.n_head, n_samp, 2):
        raise ScaleKVError(1, "terms must be a contiguous fp32 device tensor [S,H,n_samp,2]")
    if asi_out is not None and (asi_out.dtype != torch.float32 or not asi_out.is_cuda
                                or not asi_out.is_contiguous() or asi_out.numel() != 3):
        raise ScaleKVError(1, "asi_out must be a contiguous fp32 device tensor of 3 elements")
    cs, ck = shape.c(), _kv(k, shape, "k")
    wp, wb = _ws(ws)
    _check(lib().scalekv_asi(ctypes.byref(cs), _ptr(q_samp), int(n_samp), ctypes.byref(ck), int(hist_len),
                             int(cur_len), int(top_k), _ptr(terms), _ptr(asi_out), wp, wb, _stream()))


def drafter_set(asi_lk, n_drafter: int, eps: float = 1e-8):
    """scalekv_drafter_set: asi_lk is a [L][K] nested sequence of floats (host).
    Returns (is_drafter [L][K] of 0/1, z [L][K])."""
    L, K = len(asi_lk), len(asi_lk[0])
    flat = (ctypes.c_double * (L * K))(*[float(x) for row in asi_lk for x in row])
    z = (ctypes.c_double * (L * K))()
    mask = (ctypes.c_int32 * (L * K))()
    _check(lib().scalekv_drafter_set(flat, int(L), int(K), int(n_drafter), ctypes.c_double(eps), z, mask))
    return ([[int(mask[l * K + k]) for k in range(K)] for l in range(L)],
            [[float(z[l * K + k]) for k in range(K)] for l in range(L)])


def allocate_budgets(n_layer: int, n_drafter: Sequence[int], b_uniform: int, b_r0: int, delta: int,
                     b_min: int = 0):
    """scalekv_allocate_budgets -> (b_r [K], b_d, slack)."""
    K = len(n_drafter)
    nd = (ctypes.c_int32 * max(1, K))(*[int(x) for x in n_drafter])
    b_r = (ctypes.c_int32 * max(1, K))()
    b_d, slack = ctypes.c_int32(-1), ctypes.c_int64(-1)
    _check(lib().scalekv_allocate_budgets(int(n_layer), int(K), nd, ctypes.c_int64(b_uniform),
                                          ctypes.c_int64(b_r0), ctypes.c_int64(delta), ctypes.c_int64(b_min),
                                          b_r, ctypes.byref(b_d), ctypes.byref(slack)))
    return [int(b_r[k]) for k in range(K)], int(b_d.value), int(slack.value)


def policy_table(asi_lk, n_drafter: int, b_uniform: int, b_r0: int, delta: int, b_min: int = 0,
                 eps: float = 1e-8):
    """scalekv_policy_table: ASI [L][K] (host) -> (table [L][K] of per-step budgets,
    is_drafter [L][K], b_r [K], b_d, slack)."""
    L, K = len(asi_lk), len(asi_lk[0])
    flat = (ctypes.c_double * (L * K))(*[float(x) for row in asi_lk for x in row])
    table = (ctypes.c_int32 * (L * K))()
    mask = (ctypes.c_int32 * (L * K))()
    b_r = (ctypes.c_int32 * K)()
    b_d, slack = ctypes.c_int32(-1), ctypes.c_int64(-1)
    _check(lib().scalekv_policy_table(flat, int(L), int(K), int(n_drafter), ctypes.c_double(eps),
                                      ctypes.c_int64(b_uniform), ctypes.c_int64(b_r0), ctypes.c_int64(delta),
                                      ctypes.c_int64(b_min), table, mask, b_r, ctypes.byref(b_d),
                                      ctypes.byref(slack)))
    grid = lambda a: [[int(a[l * K + k]) for k in range(K)] for l in range(L)]
    return grid(table), grid(mask), [int(b_r[k]) for k in range(K)], int(b_d.value), int(slack.value)


def pyramid_budgets(n_layer: int, b_uniform: int, b_last: int) -> list:
    """scalekv_pyramid_budgets -> per-layer budgets [L]."""
    b = (ctypes.c_int32 * max(1, n_layer))()
    _check(lib().scalekv_pyramid_budgets(int(n_layer), ctypes.c_int64(b_uniform), ctypes.c_int64(b_last), b))
    return [int(b[l]) for l in range(n_layer)]


def select_positional(shape: Shape, cache_len: int, n_sink: int, n_recent: int, idx: torch.Tensor) -> int:
    """scalekv_select_positional: first n_sink and last n_recent positions -> idx [S,H,keep]; returns keep."""
    sink = max(0, min(int(n_sink), int(cache_len)))
    keep = sink + max(0, min(int(n_recent), int(cache_len) - sink))
    _idx_tensor(idx, shape, keep, "idx")
    cs = shape.c()
    out = ctypes.c_int32(-1)
    _check(lib().scalekv_select_positional(ctypes.byref(cs), int(cache_len), int(n_sink), int(n_recent),
                                           _ptr(idx), ctypes.byref(out), _stream()))
    assert out.value == keep, "the binding's shape check and the library disagree on keep"
    return int(out.value)
