"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device (so these
run without a GPU; pointers below are fake but aligned and never dereferenced)."""
import ctypes
import os
import re

import pytest
import torch

import paper_2505_19602_amd as skv
from paper_2505_19602_amd import binding as B
from paper_2505_19602_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(skv.lib_path()):
        hip_build.build(force=True)
    return skv.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "scalekv.h")).read()
    declared = set(re.findall(r"\b(scalekv_[a-z_]+)\s*\(", header))
    assert declared == set(skv.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(L, name) is not None
    assert "gfx950" in skv.version()


def _shape(**kw):
    base = dict(n_seq=1, n_head=2, head_dim=128, dtype=1, sm_scale=0.0)
    base.update(kw)
    return B._CShape(base["n_seq"], base["n_head"], base["head_dim"], base["dtype"], base["sm_scale"])


def _kv(ptr=0x10000, cap=64, d=128, heads=2):
    return B._CKv(ptr, cap * d * heads, cap * d, cap)


def _err(L):
    return L.scalekv_last_error().decode()


def test_workspace_bytes_and_shape_errors(L):
    out = ctypes.c_size_t(0)
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape()), 1000, 64, ctypes.byref(out)) == 0
    small = out.value
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape()), 4000, 64, ctypes.byref(out)) == 0
    assert out.value > small > 0
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape(head_dim=96)), 10, 1, ctypes.byref(out)) == 2
    assert "head_dim" in _err(L)
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape(dtype=7)), 10, 1, ctypes.byref(out)) == 2
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape(n_seq=0)), 10, 1, ctypes.byref(out)) == 1
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape()), -1, 1, ctypes.byref(out)) == 1
    assert L.scalekv_workspace_bytes(None, 10, 1, ctypes.byref(out)) == 1
    assert L.scalekv_workspace_bytes(ctypes.byref(_shape()), 10, 1, None) == 1


def test_score_argument_errors(L):
    s, k = _shape(), _kv()
    p = ctypes.c_void_p
    big = ctypes.c_size_t(1 << 30)
    assert L.scalekv_score(ctypes.byref(s), p(0x2000), 17, ctypes.byref(k), 10, p(0x3000), p(0x4000), big, None) == 1
    assert L.scalekv_score(ctypes.byref(s), p(0x2000), 0, ctypes.byref(k), 10, p(0x3000), p(0x4000), big, None) == 1
    assert L.scalekv_score(ctypes.byref(s), p(0), 4, ctypes.byref(k), 10, p(0x3000), p(0x4000), big, None) == 1
    assert L.scalekv_score(ctypes.byref(s), p(0x2004), 4, ctypes.byref(k), 10, p(0x3000), p(0x4000), big, None) == 1
    assert "aligned" in _err(L)
    assert L.scalekv_score(ctypes.byref(s), p(0x2000), 4, ctypes.byref(k), 65, p(0x3000), p(0x4000), big, None) == 1
    assert "capacity" in _err(L)
    assert L.scalekv_score(ctypes.byref(s), p(0x2000), 4, ctypes.byref(k), 10, p(0x3000), p(0), big, None) == 3
    assert L.scalekv_score(ctypes.byref(s), p(0x2000), 4, ctypes.byref(k), 10, p(0x3000), p(0x4000),
                           ctypes.c_size_t(16), None) == 3
    assert "needed" in _err(L)


def test_select_argument_errors(L):
    s = _shape()
    p = ctypes.c_void_p
    keep = ctypes.c_int32(-5)
    assert L.scalekv_select(ctypes.byref(s), p(0x1000), 10, -1, p(0x2000), ctypes.byref(keep), None) == 1
    assert L.scalekv_select(ctypes.byref(s), p(0), 10, 3, p(0x2000), ctypes.byref(keep), None) == 1
    assert L.scalekv_select(ctypes.byref(s), p(0x1000), 10, 3, p(0), ctypes.byref(keep), None) == 1
    # budget 0 / empty cache: legal no-ops that need no device
    assert L.scalekv_select(ctypes.byref(s), p(0), 10, 0, p(0), ctypes.byref(keep), None) == 0
    assert keep.value == 0
    assert L.scalekv_select(ctypes.byref(s), p(0), 0, 5, p(0), ctypes.byref(keep), None) == 0
    assert keep.value == 0


def test_compact_argument_errors(L):
    s = _shape()
    p = ctypes.c_void_p
    span = 64 * 128 * 2 * 2  # bytes of one fake cache
    ks, vs = _kv(0x100000), _kv(0x100000 + span)
    kd, vd = _kv(0x100000 + 2 * span), _kv(0x100000 + 3 * span)
    ok_args = lambda: (ctypes.byref(s), ctypes.byref(ks), ctypes.byref(vs), 40, p(0x9000), 10, p(0xA000), p(0xB000), 20,
                       ctypes.byref(kd), ctypes.byref(vd), None)
    a = list(ok_args()); a[5] = 41      # keep > cache_len
    assert L.scalekv_compact(*a) == 1
    a = list(ok_args()); a[5] = -1
    assert L.scalekv_compact(*a) == 1
    a = list(ok_args()); a[8] = 60      # keep + n_cur > capacity
    assert L.scalekv_compact(*a) == 1
    a = list(ok_args()); a[6] = p(0)    # k_cur NULL with n_cur > 0
    assert L.scalekv_compact(*a) == 1
    a = list(ok_args()); a[9] = ctypes.byref(ks)  # dst aliases src
    assert L.scalekv_compact(*a) == 1
    assert "overlap" in _err(L)
    a = list(ok_args()); a[10] = ctypes.byref(kd)  # v_dst aliases k_dst
    assert L.scalekv_compact(*a) == 1
    bad = B._CKv(0x100000, 10, 64 * 128, 64)   # seq stride smaller than one head
    a = list(ok_args()); a[1] = ctypes.byref(bad)
    assert L.scalekv_compact(*a) == 1


def test_attend_and_step_argument_errors(L):
    s = _shape()
    p = ctypes.c_void_p
    span = 64 * 128 * 2 * 2
    k, v = _kv(0x100000), _kv(0x100000 + span)
    kd, vd = _kv(0x100000 + 2 * span), _kv(0x100000 + 3 * span)
    assert L.scalekv_attend(ctypes.byref(s), p(0x1000), 8, ctypes.byref(k), ctypes.byref(v), 0, p(0x2000), None) == 1
    assert L.scalekv_attend(ctypes.byref(s), p(0x1000), 8, ctypes.byref(k), ctypes.byref(v), 65, p(0x2000), None) == 1
    assert L.scalekv_attend(ctypes.byref(s), p(0x1000), -1, ctypes.byref(k), ctypes.byref(v), 10, p(0x2000), None) == 1
    assert L.scalekv_attend(ctypes.byref(s), p(0x1000), 0, ctypes.byref(k), ctypes.byref(v), 10, p(0x2000), None) == 0
    win = (ctypes.c_int32 * 4)(0, 1, 2, 9)
    new_len = ctypes.c_int32(0)
    big = ctypes.c_size_t(1 << 30)

    def step(n_cur=8, n_win=4, cache_len=40, budget=10, ws=p(0x8000), ws_bytes=big, w=win):
        return L.scalekv_step(ctypes.byref(s), p(0x1000), p(0x2000), p(0x3000), n_cur, w, n_win, ctypes.byref(k),
                              ctypes.byref(v), cache_len, budget, ctypes.byref(kd), ctypes.byref(vd),
                              ctypes.byref(new_len), p(0x4000), p(0), ws, ws_bytes, None)
    assert step() == 1 and "win_idx[3]" in _err(L)          # 9 >= n_cur
    assert step(n_cur=0) == 1
    assert step(n_win=17, n_cur=32) == 1
    assert step(n_cur=16, budget=-2) == 1
    assert step(n_cur=16, ws=p(0)) == 3
    assert step(n_cur=16, ws_bytes=ctypes.c_size_t(8)) == 3
    assert step(n_cur=16, cache_len=65) == 1
    assert step(n_cur=60, budget=10) == 1 and "capacity" in _err(L)   # keep + n_cur > dst capacity


def test_step_static_checks_arguments_and_its_size_limit_before_touching_a_device(L):
    s = _shape()
    p = ctypes.c_void_p
    gib = 1 << 30
    cap = 600000                                     # 2 units x 600000 rows need ~86 MB of scratch
    k, v, kd, vd = (_kv((4 + i) * gib, cap=cap + 64) for i in range(4))
    win = (ctypes.c_int32 * 4)(0, 1, 2, 3)
    new_len = ctypes.c_int32(-1)

    def step(n_cur=8, n_win=4, cache_len=40, budget=10):
        return L.scalekv_step_static(ctypes.byref(s), p(0x1000), p(0x2000), p(0x3000), n_cur, win, n_win,
                                     ctypes.byref(k), ctypes.byref(v), cache_len, budget, ctypes.byref(kd),
                                     ctypes.byref(vd), ctypes.byref(new_len), p(0x4000), p(0), None)
    need = ctypes.c_size_t(0)
    assert L.scalekv_workspace_bytes(ctypes.byref(s), cap, 8, ctypes.byref(need)) == 0
    assert need.value > skv.STATIC_SCRATCH_BYTES
    assert step(cache_len=cap, budget=100) == 3 and "static" in _err(L)      # beyond the array: refused, nothing launched
    assert step(n_cur=0) == 1
    assert step(n_win=17, n_cur=32) == 1
    assert step(budget=-2) == 1
    assert step(n_win=4, n_cur=3) == 1               # window larger than the map
    header = open(os.path.join(ROOT, "include", "scalekv.h")).read()
    m = re.search(r"#define SCALEKV_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == skv.STATIC_SCRATCH_BYTES


def test_binding_rejects_wrong_tensors_before_calling_c():
    shape = skv.Shape(1, 2, 128, torch.bfloat16)
    q = torch.zeros(1, 2, 4, 128, dtype=torch.bfloat16)
    with pytest.raises(skv.ScaleKVError):
        skv.attend(shape, q, q, q, 4, q)          # CPU tensors are not device memory
    with pytest.raises(skv.ScaleKVError):
        skv.Shape(1, 2, 128, torch.float16).c()


# ---- entry points of the literal order of Sec. 3.3

@pytest.mark.parametrize("h,w,ph,pw", [(1, 1, 4, 4), (2, 2, 4, 4), (4, 4, 4, 4), (6, 6, 4, 4), (8, 8, 4, 4),
                                        (12, 12, 4, 4), (16, 16, 4, 4), (20, 20, 4, 4), (24, 24, 4, 4),
                                        (32, 32, 4, 4), (40, 40, 4, 4), (48, 48, 4, 4), (64, 64, 4, 4),
                                        (6, 10, 4, 4), (7, 5, 2, 3), (64, 64, 3, 5), (33, 17, 4, 4), (5, 64, 8, 8)])
def test_window_centroids_match_the_oracle(L, h, w, ph, pw):
    # host-only integer work: the library's result is compared with the oracle's on the CPU
    import oracle
    assert skv.window_centroids(h, w, ph, pw) == oracle.window_centroids(h, w, ph, pw).tolist()


def test_window_centroids_argument_errors(L):
    buf = (ctypes.c_int32 * 16)()
    n = ctypes.c_int32(0)
    assert L.scalekv_window_centroids(0, 4, 4, 4, buf, ctypes.byref(n)) == 1
    assert L.scalekv_window_centroids(4, 4, 0, 4, buf, ctypes.byref(n)) == 1
    assert L.scalekv_window_centroids(4, 4, 4, 4, None, ctypes.byref(n)) == 1
    assert L.scalekv_window_centroids(4, 4, 4, 4, buf, None) == 1
    assert L.scalekv_window_centroids(65536, 65536, 4, 4, buf, ctypes.byref(n)) == 2


def test_select_window_argument_errors(L):
    s = _shape()
    p = ctypes.c_void_p
    keep = ctypes.c_int32(-5)
    f = (ctypes.c_int32 * 3)(1, 4, 9)
    call = lambda budget=3, forced=f, n_forced=3, pool_w=1, scores=p(0x1000), idx=p(0x2000), cache_len=10: \
        L.scalekv_select_window(ctypes.byref(s), scores, cache_len, budget, forced, n_forced, pool_w, idx,
                                ctypes.byref(keep), None)
    assert call(budget=-1) == 1
    assert call(pool_w=2) == 1 and "pool_w" in _err(L)
    assert call(pool_w=0) == 1
    assert call(pool_w=33) == 1
    assert call(n_forced=17) == 1
    assert call(forced=None) == 1
    assert call(forced=(ctypes.c_int32 * 3)(1, 4, 10)) == 1 and "forced[2]" in _err(L)
    assert call(forced=(ctypes.c_int32 * 3)(1, 4, 4)) == 1 and "repeats" in _err(L)
    assert call(scores=p(0)) == 1
    assert call(idx=p(0)) == 1
    # nothing to select: legal no-op that needs no device
    assert call(budget=0, n_forced=0, scores=p(0), idx=p(0)) == 0 and keep.value == 0


def test_step_append_first_argument_errors(L):
    s = _shape()
    p = ctypes.c_void_p
    span = 64 * 128 * 2 * 2
    k, v = _kv(0x100000), _kv(0x100000 + span)
    kn, vn = _kv(0x100000 + 2 * span), _kv(0x100000 + 3 * span)
    win = (ctypes.c_int32 * 4)(0, 1, 2, 9)
    keep, moved = ctypes.c_int32(0), ctypes.c_int32(0)
    big = ctypes.c_size_t(1 << 30)

    def step(n_cur=16, n_win=4, pool_w=1, cache_len=40, budget=10, ws=p(0x8000), ws_bytes=big, w=win,
             kc=k, vc=v, k_next=kn):
        return L.scalekv_step_append_first(
            ctypes.byref(s), p(0x1000), p(0x2000), p(0x3000), n_cur, w, n_win, pool_w, ctypes.byref(kc),
            ctypes.byref(vc), cache_len, budget, ctypes.byref(k_next), ctypes.byref(vn), ctypes.byref(keep),
            ctypes.byref(moved), p(0x4000), p(0), ws, ws_bytes, None)
    assert step(n_cur=8) == 1 and "win_idx[3]" in _err(L)
    assert step(n_cur=0) == 1
    assert step(budget=-1) == 1
    assert step(pool_w=4) == 1
    assert step(n_win=17, n_cur=20) == 1
    assert step(cache_len=50) == 1 and "capacity" in _err(L)      # 50 + 16 rows do not fit 64
    assert step(ws=p(0)) == 3
    assert step(ws_bytes=ctypes.c_size_t(8)) == 3
    assert step(n_win=0) == 1 and "window" in _err(L)             # a ranking without window rows
    assert step(vc=k) == 1 and "overlap" in _err(L)
    assert step(k_next=k) == 1 and "overlap" in _err(L)
    assert step(w=(ctypes.c_int32 * 4)(0, 1, 2, 2)) == 1 and "repeats" in _err(L)


def test_step_and_compact_reject_inputs_that_overlap_the_destination(L):
    s = _shape()
    p = ctypes.c_void_p
    big = ctypes.c_size_t(1 << 30)
    src_k, src_v = _kv(0x100000), _kv(0x200000)
    dst_k, dst_v = _kv(0x300000), _kv(0x400000)            # 64 rows x 128 x 2 heads x 2 B = 32 KiB each
    win = (ctypes.c_int32 * 1)(0)
    new_len = ctypes.c_int32(-1)
    def step(q, kc, vc, out):
        return L.scalekv_step(ctypes.byref(s), p(q), p(kc), p(vc), 8, win, 1, ctypes.byref(src_k), ctypes.byref(src_v),
                              20, 5, ctypes.byref(dst_k), ctypes.byref(dst_v), ctypes.byref(new_len), p(out), None,
                              p(0x800000), big, None)
    assert step(0x300000 + 4096, 0x600000, 0x700000, 0x900000) == 1 and "overlaps a destination" in _err(L)
    assert step(0x500000, 0x400000, 0x700000, 0x900000) == 1
    assert step(0x500000, 0x600000, 0x300000 - 256, 0x900000) == 1      # its last bytes reach into k_dst
    assert step(0x500000, 0x600000, 0x700000, 0x400000 + 32 * 1024 - 16) == 1
    assert L.scalekv_compact(ctypes.byref(s), ctypes.byref(src_k), ctypes.byref(src_v), 20, None, 5, p(0x300000), p(0x700000),
                             8, ctypes.byref(dst_k), ctypes.byref(dst_v), None) == 1
    assert "overlap a destination" in _err(L)


def test_step_append_first_rejects_inputs_that_overlap_the_next_cache(L):
    # the final pruning writes k_next / v_next after the attention has stored `out`
    s = _shape()
    p = ctypes.c_void_p
    big = ctypes.c_size_t(1 << 30)
    k_cache, v_cache = _kv(0x100000), _kv(0x200000)
    k_next, v_next = _kv(0x300000), _kv(0x400000)
    win = (ctypes.c_int32 * 1)(0)
    keep, moved = ctypes.c_int32(-1), ctypes.c_int32(-1)

    def step(q, kc, vc, out, budget=5):
        return L.scalekv_step_append_first(ctypes.byref(s), p(q), p(kc), p(vc), 8, win, 1, 1, ctypes.byref(k_cache),
                                           ctypes.byref(v_cache), 20, budget, ctypes.byref(k_next),
                                           ctypes.byref(v_next), ctypes.byref(keep), ctypes.byref(moved), p(out), None,
                                           p(0x800000), big, None)
    assert step(0x500000, 0x600000, 0x700000, 0x300000 + 1024) == 1 and "next-cache" in _err(L)     # out in k_next
    assert step(0x400000 + 512, 0x600000, 0x700000, 0x900000) == 1                                    # q in v_next
    assert step(0x500000, 0x600000, 0x300000, 0x900000) == 1                                          # v_cur in k_next

