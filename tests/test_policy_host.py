"""Host-side parts of the offline policy in the C ABI (drafter set of Eq. 3, budget
allocation of Eq. 4, pyramid budgets of Sec. 4.1) against the oracle, and the argument
checks of the policy entry points.  No GPU needed: nothing here launches a kernel."""
import ctypes
import os

import numpy as np
import pytest

import oracle
import paper_2505_19602_amd as skv
from paper_2505_19602_amd import binding as B
from paper_2505_19602_amd import build as hip_build


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(skv.lib_path()):
        hip_build.build(force=True)
    return skv.lib()


def _err(L):
    return L.scalekv_last_error().decode()


@pytest.mark.parametrize("seed", range(5))
def test_drafter_set_matches_the_oracle(L, seed):
    rng = np.random.default_rng(seed)
    nl, nk = int(rng.integers(2, 41)), int(rng.integers(1, 14))
    asi = rng.uniform(0.0, 1.0, size=(nl, nk)) * rng.uniform(0.01, 10, size=(1, nk))
    for n_d in (0, 1, nl, nl * nk // 3, nl * nk, nl * nk + 5):
        mask, z = skv.drafter_set(asi.tolist(), n_d, eps=1e-8)
        zo = oracle.zscores(asi, eps=1e-8)
        assert np.allclose(np.array(z), zo, rtol=1e-12, atol=1e-12)
        # the set is a function of the ranking; compare where the oracle's own Z separates
        assert np.array_equal(np.array(mask), oracle.drafters(zo, n_d))


def test_drafter_set_ties_and_constant_scales(L):
    mask, z = skv.drafter_set([[0.5, 0.5], [0.5, 0.5], [0.5, 0.5]], 4, eps=1e-8)
    assert np.array_equal(np.array(mask), oracle.drafters(np.zeros((3, 2)), 4))
    assert mask == [[1, 1], [1, 0], [1, 0]] and np.all(np.array(z) == 0)
    mask, z = skv.drafter_set([[1.0], [1.0]], 1, eps=0.0)          # sigma + eps == 0
    assert np.all(np.array(z) == 0) and mask == [[1], [0]]


def test_drafter_set_argument_errors(L):
    d = ctypes.c_double * 4
    m = (ctypes.c_int32 * 4)()
    assert L.scalekv_drafter_set(d(1, 2, 3, 4), 0, 4, 1, ctypes.c_double(0), None, m) == 1
    assert L.scalekv_drafter_set(d(1, 2, 3, 4), 2, 2, -1, ctypes.c_double(0), None, m) == 1
    assert L.scalekv_drafter_set(d(1, 2, 3, 4), 2, 2, 1, ctypes.c_double(-1), None, m) == 1
    assert L.scalekv_drafter_set(None, 2, 2, 1, ctypes.c_double(0), None, m) == 1
    assert L.scalekv_drafter_set(d(1, 2, 3, 4), 2, 2, 1, ctypes.c_double(0), None, None) == 1
    assert L.scalekv_drafter_set(d(1, float("nan"), 3, 4), 2, 2, 1, ctypes.c_double(0), None, m) == 1
    assert "finite" in _err(L)


@pytest.mark.parametrize("seed", range(8))
def test_allocate_budgets_matches_the_oracle(L, seed):
    rng = np.random.default_rng(100 + seed)
    nl, nk = int(rng.integers(1, 48)), int(rng.integers(1, 14))
    n_d = rng.integers(0, nl + 1, size=nk); n_d[-1] = max(1, n_d[-1])
    bu, br0 = int(rng.integers(20, 2000)), int(rng.integers(0, 200))
    delta, b_min = int(rng.integers(0, 40)), int(rng.integers(0, 5))
    want = oracle.budgets(nl, n_d, bu, br0, delta, b_min)
    if want is None:
        with pytest.raises(skv.ScaleKVError):
            skv.allocate_budgets(nl, n_d.tolist(), bu, br0, delta, b_min)
        return
    b_r, b_d, slack = skv.allocate_budgets(nl, n_d.tolist(), bu, br0, delta, b_min)
    assert b_r == want[0].tolist() and b_d == want[1] and slack == want[2]


def test_allocate_budgets_with_the_papers_numbers(L):
    b_r, b_d, slack = skv.allocate_budgets(32, [8] * 13, 650, 600, 70)
    assert (b_r, b_d, slack) == (oracle.budgets(32, [8] * 13, 650, 600, 70)[0].tolist(), 2073, 88)


def test_allocate_budgets_argument_errors(L):
    nd = (ctypes.c_int32 * 2)(1, 1)
    br = (ctypes.c_int32 * 2)()
    bd, sl = ctypes.c_int32(), ctypes.c_int64()
    i64 = ctypes.c_int64
    call = lambda *a: L.scalekv_allocate_budgets(*a)
    ok = (4, 2, nd, i64(10), i64(5), i64(1), i64(0), br, ctypes.byref(bd), ctypes.byref(sl))
    assert call(*ok) == 0
    assert call(0, 2, nd, i64(10), i64(5), i64(1), i64(0), br, ctypes.byref(bd), None) == 1
    assert call(4, 2, None, i64(10), i64(5), i64(1), i64(0), br, ctypes.byref(bd), None) == 1
    assert call(4, 2, nd, i64(-1), i64(5), i64(1), i64(0), br, ctypes.byref(bd), None) == 1
    assert call(4, 2, nd, i64(10), i64(50), i64(0), i64(0), br, ctypes.byref(bd), None) == 1
    assert "exceed" in _err(L)
    assert call(4, 2, (ctypes.c_int32 * 2)(0, 0), i64(10), i64(5), i64(0), i64(0), br, ctypes.byref(bd), None) == 1
    assert call(4, 2, (ctypes.c_int32 * 2)(5, 0), i64(10), i64(5), i64(0), i64(0), br, ctypes.byref(bd), None) == 1
    assert call(4, 2, nd, i64(10), i64(5), i64(1), i64(0), br, ctypes.byref(bd), None) == 0   # slack optional


def _oracle_table(asi, n_d, bu, br0, delta, b_min, eps=1e-8):
    """Eq. 3 then Eq. 4 through the oracle, and the budget of every (layer, scale) pair."""
    mask = oracle.drafters(oracle.zscores(asi, eps=eps), n_d)
    sol = oracle.budgets(asi.shape[0], mask.sum(axis=0), bu, br0, delta, b_min)
    if sol is None:
        return None
    b_r, b_d, slack = sol
    return np.where(mask == 1, b_d, b_r[None, :]), mask, b_r, b_d, slack


@pytest.mark.parametrize("seed", range(8))
def test_policy_table_matches_the_oracle(L, seed):
    rng = np.random.default_rng(300 + seed)
    nl, nk = int(rng.integers(2, 41)), int(rng.integers(1, 14))
    asi = rng.uniform(0.0, 1.0, size=(nl, nk)) * rng.uniform(0.01, 10, size=(1, nk))
    n_d = int(rng.integers(1, nl * nk + 1))
    bu, br0 = int(rng.integers(50, 2000)), int(rng.integers(0, 300))
    delta, b_min = int(rng.integers(0, 40)), int(rng.integers(0, 5))
    want = _oracle_table(asi, n_d, bu, br0, delta, b_min)
    if want is None:
        with pytest.raises(skv.ScaleKVError):
            skv.policy_table(asi.tolist(), n_d, bu, br0, delta, b_min)
        return
    table, mask, b_r, b_d, slack = skv.policy_table(asi.tolist(), n_d, bu, br0, delta, b_min)
    assert np.array_equal(np.array(table), want[0]) and np.array_equal(np.array(mask), want[1])
    assert b_r == want[2].tolist() and (b_d, slack) == (want[3], want[4])
    # Eq. 4 itself: the budgets handed out add up to the uniform total, short by the slack
    assert int(np.array(table).sum()) + slack == bu * nl * nk


def test_policy_table_with_the_papers_numbers(L):
    """32 layers, 13 scales, 104 drafter pairs, B_uniform 650, B_r(0) 600, delta 70 (Sec. 4.1 /
    Appendix): whatever the ASI values, refiners follow the clamped line and Eq. 4 balances."""
    rng = np.random.default_rng(7)
    asi = rng.uniform(0.0, 1.0, size=(32, 13))
    table, mask, b_r, b_d, slack = skv.policy_table(asi.tolist(), 104, 650, 600, 70)
    assert b_r == [530, 460, 390, 320, 250, 180, 110, 40, 0, 0, 0, 0, 0]
    assert int(np.array(mask).sum()) == 104
    assert int(np.array(table).sum()) + slack == 650 * 32 * 13 and 0 <= slack < 104
    want = _oracle_table(asi, 104, 650, 600, 70, 0)
    assert np.array_equal(np.array(table), want[0])


def test_policy_table_argument_errors(L):
    d = ctypes.c_double * 4
    t = (ctypes.c_int32 * 4)()
    i64 = ctypes.c_int64
    args = lambda asi, nl, nk, nd, tab: (asi, nl, nk, nd, ctypes.c_double(1e-8), i64(100), i64(50), i64(10), i64(0),
                                        tab, None, None, None, None)
    assert L.scalekv_policy_table(*args(d(1, 2, 3, 4), 2, 2, 1, t)) == 0
    assert L.scalekv_policy_table(*args(d(1, 2, 3, 4), 2, 2, 1, None)) == 1
    assert L.scalekv_policy_table(*args(d(1, 2, 3, 4), 2, 2, 0, t)) == 1      # nothing could take the pool
    assert L.scalekv_policy_table(*args(None, 2, 2, 1, t)) == 1
    assert L.scalekv_policy_table(*args(d(1, 2, 3, 4), 0, 2, 1, t)) == 1
    # refiners alone above the total
    assert L.scalekv_policy_table(d(1, 2, 3, 4), 2, 2, 1, ctypes.c_double(1e-8), i64(10), i64(500), i64(0), i64(0),
                                  t, None, None, None, None) == 1
    assert "exceed" in _err(L)


@pytest.mark.parametrize("nl,bu,bl", [(1, 7, 7), (2, 9, 4), (7, 100, 30), (8, 100, 30), (32, 650, 100), (40, 649, 0), (5, 10, 10)])
def test_pyramid_budgets_match_the_oracle(L, nl, bu, bl):
    assert skv.pyramid_budgets(nl, bu, bl) == oracle.pyramid(nl, bu, bl).tolist()


def test_pyramid_and_positional_argument_errors(L):
    b = (ctypes.c_int32 * 4)()
    i64 = ctypes.c_int64
    assert L.scalekv_pyramid_budgets(0, i64(10), i64(5), b) == 1
    assert L.scalekv_pyramid_budgets(4, i64(10), i64(11), b) == 1
    assert L.scalekv_pyramid_budgets(4, i64(10), i64(-1), b) == 1
    assert L.scalekv_pyramid_budgets(4, i64(10), i64(5), None) == 1
    s = B._CShape(1, 2, 128, 1, 0.0)
    keep = ctypes.c_int32(-1)
    p = ctypes.c_void_p
    assert L.scalekv_select_positional(ctypes.byref(s), 10, -1, 2, p(0x1000), ctypes.byref(keep), None) == 1
    assert L.scalekv_select_positional(ctypes.byref(s), 10, 1, -2, p(0x1000), ctypes.byref(keep), None) == 1
    assert L.scalekv_select_positional(ctypes.byref(s), -1, 1, 2, p(0x1000), ctypes.byref(keep), None) == 1
    assert L.scalekv_select_positional(ctypes.byref(s), 10, 1, 2, p(0), ctypes.byref(keep), None) == 1
    # nothing to keep: no launch, keep reported
    assert L.scalekv_select_positional(ctypes.byref(s), 10, 0, 0, p(0), ctypes.byref(keep), None) == 0
    assert keep.value == 0


def test_asi_argument_errors(L):
    s = B._CShape(1, 2, 128, 1, 0.0)
    k = B._CKv(0x10000, 64 * 128 * 2, 64 * 128, 64)
    p = ctypes.c_void_p
    big = ctypes.c_size_t(1 << 30)
    call = lambda *a: L.scalekv_asi(ctypes.byref(s), *a)
    assert call(p(0x2000), 0, ctypes.byref(k), 10, 4, 2, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), skv.MAX_ASI_SAMPLES + 1, ctypes.byref(k), 10, 4, 2, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), 10, 4, -1, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), -1, 4, 2, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), 0, 0, 2, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), 60, 10, 2, p(0x3000), None, p(0x4000), big, None) == 1   # beyond capacity
    assert "capacity" in _err(L)
    assert call(p(0), 4, ctypes.byref(k), 10, 4, 2, p(0x3000), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), 10, 4, 2, p(0), None, p(0x4000), big, None) == 1
    assert call(p(0x2000), 4, ctypes.byref(k), 10, 4, 2, p(0x3000), None, p(0), big, None) == 3
    assert call(p(0x2000), 4, ctypes.byref(k), 10, 4, 2, p(0x3000), None, p(0x4000), ctypes.c_size_t(16), None) == 3
