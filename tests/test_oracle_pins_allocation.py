"""Pins for the oracle of the offline policy (oracle/allocation.c): ASI (Eq. 2),
Z-score and drafter set (Eq. 3), budget allocation (Eq. 4) and the comparison
policies of Sec. 4.1.  Closed forms, invariants, hand-worked values and brute
force on tiny inputs; none retypes the oracle's loops."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            out[k.strip()] = v.strip()
    return out


# ------------------------------------------------------------------ Eq. 2 --

def test_asi_identical_keys_give_the_counting_closed_form():
    # every key equal -> uniform attention: cur = n_cur / n, top-K' of history = K' / n
    rng = np.random.default_rng(0)
    d, hist, cur, kp = 8, 11, 5, 3
    k = np.tile(rng.normal(size=(1, 1, d)), (1, hist + cur, 1))
    q = rng.normal(size=(1, 4, d))
    c, t = oracle.asi_terms(q, k, hist, kp)
    assert np.allclose(c, cur / (hist + cur), rtol=0, atol=1e-14)
    assert np.allclose(t, kp / (hist + cur), rtol=0, atol=1e-14)


def test_asi_terms_complete_each_other_when_top_k_covers_the_history():
    # attention rows sum to 1, so current mass + all of the history mass = 1
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=(3, 6, 16)), rng.normal(size=(3, 40, 16)) * 2
    for kp in (25, 26, 1000):
        c, t = oracle.asi_terms(q, k, 25, kp)
        assert np.allclose(c + t, 1.0, rtol=0, atol=1e-13)


def test_asi_top_sum_is_monotone_concave_in_k_and_starts_at_the_largest_weight():
    rng = np.random.default_rng(2)
    q, k = rng.normal(size=(2, 5, 8)) * 3, rng.normal(size=(2, 30, 8))
    hist = 22
    tops = np.stack([oracle.asi_terms(q, k, hist, kp)[1] for kp in range(0, hist + 1)])
    assert np.all(tops[0] == 0)
    inc = np.diff(tops, axis=0)            # the kp-th largest weight
    assert np.all(inc > 0) and np.all(np.diff(inc, axis=0) <= 1e-15)
    # K' = 1 is the largest history weight of a textbook softmax row
    lg = np.einsum("uqd,ukd->uqk", q, k) / np.sqrt(8)
    p = np.exp(lg - lg.max(-1, keepdims=True)); p /= p.sum(-1, keepdims=True)
    assert np.allclose(tops[1], p[..., :hist].max(-1), rtol=1e-13)


def test_asi_top_sum_equals_the_best_subset_by_brute_force():
    rng = np.random.default_rng(3)
    d, hist, cur, kp = 4, 7, 3, 3
    q, k = rng.normal(size=(1, 2, d)) * 2, rng.normal(size=(1, hist + cur, d))
    c, t = oracle.asi_terms(q, k, hist, kp, scale=0.7)
    lg = np.einsum("uqd,ukd->uqk", q, k) * 0.7
    p = np.exp(lg); p /= p.sum(-1, keepdims=True)
    for i in range(2):
        best = max(sum(p[0, i, j] for j in sub) for sub in itertools.combinations(range(hist), kp))
        assert np.isclose(t[0, i], best, rtol=1e-13)
        assert np.isclose(c[0, i], p[0, i, hist:].sum(), rtol=1e-13)


def test_asi_history_and_current_are_not_swapped():
    # a query aligned with one current-map key: all mass on the current map, none in history
    d, hist, cur = 8, 6, 4
    k = np.zeros((1, hist + cur, d)); k[0, hist + 2, 0] = 50.0
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 50.0
    c, t = oracle.asi_terms(q, k, hist, 2)
    assert c[0, 0] > 1 - 1e-12 and t[0, 0] < 1e-12
    # and aligned with one history key: the top-1 history weight is everything
    k = np.zeros((1, hist + cur, d)); k[0, 3, 0] = 50.0
    c, t = oracle.asi_terms(q, k, hist, 1)
    assert c[0, 0] < 1e-12 and t[0, 0] > 1 - 1e-12


def test_asi_is_the_product_of_the_two_means_not_the_mean_of_products():
    c = np.array([0.2, 0.8]); t = np.array([0.5, 0.1])
    assert np.isclose(oracle.asi(c, t), 0.5 * 0.3)      # mean of products would be 0.09
    assert oracle.asi(np.zeros(0), np.zeros(0)) == 0.0


# ------------------------------------------------------------------ Eq. 3 --

def test_zscores_have_zero_mean_and_unit_population_deviation_per_scale():
    rng = np.random.default_rng(4)
    a = rng.uniform(size=(12, 5)) * np.array([1, 10, 100, 0.01, 3])
    z = oracle.zscores(a, eps=0.0)
    assert np.allclose(z.mean(0), 0, atol=1e-12)
    assert np.allclose((z ** 2).mean(0), 1, rtol=1e-12)       # divisor L, not L - 1
    # normalisation is within a scale: rescaling one scale's ASI leaves every Z unchanged
    b = a.copy(); b[:, 2] = 7 * b[:, 2] + 3
    assert np.allclose(oracle.zscores(b, eps=0.0), z, atol=1e-10)


def test_zscore_eps_guards_a_constant_scale():
    a = np.ones((6, 2)); a[:, 1] = np.arange(6)
    z = oracle.zscores(a, eps=1e-8)
    assert np.all(z[:, 0] == 0) and np.all(np.isfinite(z))
    # hand value: scale 1 has mean 2.5, population variance 35/12
    assert np.isclose(z[0, 1], -2.5 / (np.sqrt(35 / 12) + 1e-8), rtol=1e-14)


def test_drafters_are_the_lowest_z_pairs_over_all_layers_and_scales():
    rng = np.random.default_rng(5)
    z = rng.normal(size=(8, 6))
    for n_d in (0, 1, 7, 20, 48, 100):
        m = oracle.drafters(z, n_d)
        n = min(n_d, 48)
        assert m.sum() == n
        if 0 < n < 48:
            assert z[m == 1].max() < z[m == 0].min()


def test_drafter_ties_go_to_the_lower_scale_then_the_lower_layer():
    z = np.zeros((3, 2))                      # all equal
    m = oracle.drafters(z, 4)
    # scan order: scale 0 layers 0,1,2 then scale 1 layer 0
    assert m.tolist() == [[1, 1], [1, 0], [1, 0]]


def test_low_asi_means_drafter():
    # Sec. 3.3: low ASI = attention spread over the prefix = drafter.  Layer 0 spreads, layer 1 focuses.
    asi = np.array([[0.01, 0.02], [0.5, 0.6], [0.4, 0.7]])
    m = oracle.drafters(oracle.zscores(asi), 2)
    assert m.tolist() == [[1, 1], [0, 0], [0, 0]]


# ------------------------------------------------------------------ Eq. 4 --

def test_budgets_reproduce_the_hand_worked_example_with_the_papers_numbers():
    g = _golden("budget_worked_example.txt")
    L, K, nd = int(g["layers"]), int(g["scales"]), int(g["drafters_per_scale"])
    b_r, b_d, slack = oracle.budgets(L, [nd] * K, int(g["b_uniform"]), int(g["b_r0"]), int(g["delta"]))
    assert b_r.tolist() == [int(x) for x in g["b_r"].split()]
    assert b_d == int(g["b_d"]) and slack == int(g["slack"])


@pytest.mark.parametrize("seed", range(6))
def test_budgets_satisfy_the_memory_constraint_up_to_the_stated_slack(seed):
    rng = np.random.default_rng(seed)
    L, K = int(rng.integers(2, 40)), int(rng.integers(1, 14))
    n_d = rng.integers(0, L + 1, size=K); n_d[0] = max(n_d[0], 1)
    bu, br0, delta = int(rng.integers(50, 900)), int(rng.integers(10, 50)), int(rng.integers(0, 8))
    b_r, b_d, slack = oracle.budgets(L, n_d, bu, br0, delta, b_min=2)
    lhs = sum(int(n_d[k]) * b_d + (L - int(n_d[k])) * int(b_r[k]) for k in range(K))
    assert lhs + slack == bu * L * K
    assert 0 <= slack < n_d.sum()
    assert np.all(np.diff(b_r) <= 0) and b_r.min() >= 2       # linear decay, held at the floor
    assert b_r[0] == max(2, br0 - delta)                       # k counts from 1


def test_budgets_without_decay_and_with_equal_refiners_are_uniform():
    b_r, b_d, slack = oracle.budgets(10, [3] * 5, 100, 100, 0)
    assert b_r.tolist() == [100] * 5 and b_d == 100 and slack == 0


def test_budgets_report_when_there_is_no_solution():
    assert oracle.budgets(4, [0, 0], 10, 5, 0) is None          # nobody to take the pool
    assert oracle.budgets(4, [1, 1], 10, 50, 0) is None         # refiners alone exceed the total


# ----------------------------------------------------- comparison policies --

def test_positional_policies():
    assert oracle.positional(10, 0, 4).tolist() == [6, 7, 8, 9]            # sliding window
    assert oracle.positional(10, 2, 3).tolist() == [0, 1, 7, 8, 9]         # sinks + recent
    assert oracle.positional(5, 3, 4).tolist() == [0, 1, 2, 3, 4]          # ranges meet: each once
    assert oracle.positional(5, 0, 0).tolist() == []
    assert oracle.positional(0, 2, 2).tolist() == []
    for n, s, r in itertools.product(range(0, 9), range(0, 5), range(0, 5)):
        got = oracle.positional(n, s, r)
        assert len(got) == min(n, s + r) and np.all(np.diff(got) > 0)


@pytest.mark.parametrize("L,bu,bl", [(8, 100, 30), (7, 100, 30), (32, 650, 100), (1, 50, 50), (2, 9, 4), (5, 10, 10)])
def test_pyramid_budgets_fall_linearly_and_keep_the_mean(L, bu, bl):
    b = oracle.pyramid(L, bu, bl)
    assert b.sum() == L * bu
    assert np.all(np.diff(b) <= 0)
    if L > 1:
        assert b[-1] == bl and b[0] == 2 * bu - bl
        line = (2 * bu - bl) - (2 * bu - 2 * bl) * np.arange(L) / (L - 1)
        assert np.all(np.abs(b - line) < 1)
