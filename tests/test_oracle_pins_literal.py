"""Pins for the oracle of the literal reading of Sec. 3.3 (append, attend, score
over history and the current map, pool, keep window + top-budget): closed forms,
library routines, brute force on tiny inputs, hand-built cases.  None retypes
the oracle's loops."""
import math

import numpy as np
import pytest
import torch

import oracle


def _sdpa(q, k, v):
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))
    return torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v)).numpy()


# ------------------------------------------------------ window centroids --

def test_centroids_of_odd_patches_are_the_exact_middles():
    # 12 x 12 map, 4 x 4 patches of 3 x 3 tokens: the middle token of each patch
    got = oracle.window_centroids(12, 12, 4, 4)
    want = [r * 12 + c for r in (1, 4, 7, 10) for c in (1, 4, 7, 10)]
    assert got.tolist() == want


def test_centroids_typical_window_is_16_tokens_and_even_patches_take_the_upper_left_middle():
    # Sec. 3.3: the window typically has 16 tokens -> a 4 x 4 grid.  On the 64 x 64 map the
    # patches are 16 x 16 and four tokens are equally central; the stated rule takes row 7, col 7.
    got = oracle.window_centroids(64, 64, 4, 4)
    assert len(got) == 16
    assert got.tolist() == [r * 64 + c for r in (7, 23, 39, 55) for c in (7, 23, 39, 55)]


def test_centroids_small_maps_use_every_token():
    assert oracle.window_centroids(1, 1).tolist() == [0]
    assert oracle.window_centroids(2, 2).tolist() == [0, 1, 2, 3]
    assert oracle.window_centroids(4, 4).tolist() == list(range(16))
    assert len(oracle.window_centroids(2, 6, 4, 4)) == 8


@pytest.mark.parametrize("h,w,ph,pw", [(6, 6, 4, 4), (6, 10, 4, 4), (10, 6, 4, 4), (10, 10, 4, 4), (20, 20, 4, 4),
                                      (7, 5, 2, 3), (11, 13, 3, 5), (48, 48, 4, 4)])
def test_centroids_minimise_distance_to_the_patch_centre(h, w, ph, pw):
    got = oracle.window_centroids(h, w, ph, pw)
    assert np.all(np.diff(got) > 0)
    PH, PW = min(ph, h), min(pw, w)
    rb = [a * h // PH for a in range(PH + 1)]
    cb = [b * w // PW for b in range(PW + 1)]
    seen = set()
    for t in got:
        r, c = divmod(int(t), w)
        a = max(i for i in range(PH) if rb[i] <= r)
        b = max(i for i in range(PW) if cb[i] <= c)
        assert (a, b) not in seen          # one token per patch
        seen.add((a, b))
        cy, cx = (rb[a] + rb[a + 1]) / 2.0, (cb[b] + cb[b + 1]) / 2.0
        rr, cc = np.meshgrid(np.arange(rb[a], rb[a + 1]), np.arange(cb[b], cb[b + 1]), indexing="ij")
        dist = np.hypot(rr + 0.5 - cy, cc + 0.5 - cx)
        assert np.isclose(np.hypot(r + 0.5 - cy, c + 0.5 - cx), dist.min())
        # among the equally near, the first in raster order
        near = np.argwhere(np.isclose(dist, dist.min()))
        assert (r - rb[a], c - cb[b]) == tuple(near[0])
    assert len(seen) == PH * PW


# ---------------------------------------------------------------- pooling --

def test_pool_width_one_is_identity_and_odd_widths_match_library_convolution():
    rng = np.random.default_rng(0)
    s = rng.random((3, 37))
    assert np.array_equal(oracle.pool(s, 1), s)
    for w in (3, 5, 9):
        want = np.stack([np.convolve(row, np.ones(w) / w, mode="same") for row in s])
        np.testing.assert_allclose(oracle.pool(s, w), want, rtol=0, atol=1e-15)


def test_pool_constant_scores_closed_form():
    # zeros beyond both ends, divisor always pool_w: edges see (r + 1 + i) / w of the constant
    out = oracle.pool(np.full((1, 10), 3.0), 5)[0]
    np.testing.assert_allclose(out, [3 * 3 / 5, 3 * 4 / 5] + [3.0] * 6 + [3 * 4 / 5, 3 * 3 / 5], atol=1e-15)


def test_pool_log_is_the_logarithm_of_the_pooled_scores_and_survives_underflow():
    rng = np.random.default_rng(3)
    s = rng.random((2, 41)) + 1e-3
    for w in (1, 3, 7, 31):
        np.testing.assert_allclose(oracle.pool_log(np.log(s), w), np.log(oracle.pool(s, w)), rtol=0, atol=1e-13)
    # log-scores far below what exp() can represent: shifting all of them by a constant shifts the
    # pooled value by the same constant (the average is homogeneous), so the result is known from a
    # representable case
    ls = np.log(s) - 5000.0
    assert np.all(np.exp(ls) == 0.0)
    np.testing.assert_allclose(oracle.pool_log(ls, 5), np.log(oracle.pool(s, 5)) - 5000.0, rtol=0, atol=1e-9)
    # a window that holds nothing but zero scores stays at log 0
    ls2 = np.full((1, 9), -np.inf); ls2[0, 8] = 0.0
    out = oracle.pool_log(ls2, 3)[0]
    assert np.all(np.isneginf(out[:7])) and np.isclose(out[7], -math.log(3.0)) and np.isclose(out[8], -math.log(3.0))


def test_literal_step_ranks_on_pooled_log_scores_same_choice_as_pooled_scores():
    rng = np.random.default_rng(27)
    for trial in range(10):
        q, kc, vc, ks, vs = _rand_case(100 + trial)
        budget, w = int(rng.integers(1, 9)), int(rng.choice([1, 3, 5]))
        r = oracle.step_append_first(q, kc, vc, [4], ks, vs, budget, pool_w=w)
        L = ks.shape[1]
        want = oracle.select_forced(r["scores"], budget, [L + 4])
        assert np.array_equal(r["idx"], want)
        np.testing.assert_allclose(r["log_scores"], np.log(r["scores"]), rtol=0, atol=1e-12)


# ------------------------------------------------- selection with a window --

def test_select_forced_without_forced_positions_is_plain_select():
    rng = np.random.default_rng(1)
    s = rng.random((4, 25))
    for b in (0, 1, 7, 25, 30):
        assert np.array_equal(oracle.select_forced(s, b, []), oracle.select(s, b))


def test_select_forced_against_sorting_on_tiny_inputs():
    rng = np.random.default_rng(2)
    for trial in range(200):
        L = int(rng.integers(1, 12))
        s = rng.integers(0, 4, size=(1, L)).astype(float)       # many ties
        n_f = int(rng.integers(0, L + 1))
        forced = sorted(rng.choice(L, size=n_f, replace=False).tolist())
        b = int(rng.integers(0, L + 2))
        rest = [i for i in range(L) if i not in forced]
        ranked = sorted(rest, key=lambda i: (-s[0, i], i))       # score descending, index ascending
        want = sorted(forced + ranked[:min(b, len(rest))])
        assert oracle.select_forced(s, b, forced)[0].tolist() == want


def test_select_forced_positions_do_not_use_up_the_budget():
    s = np.array([[9.0, 8.0, 7.0, 1.0, 2.0, 3.0]])
    # positions 0 and 1 are forced and also score highest: the budget of 2 still buys 2 others
    assert oracle.select_forced(s, 2, [0, 1])[0].tolist() == [0, 1, 2, 5]
    # forced positions with the lowest scores stay
    assert oracle.select_forced(s, 1, [3])[0].tolist() == [0, 3]
    assert oracle.select_forced(s, 0, [3, 4])[0].tolist() == [3, 4]


# ---------------------------------------------------------- the literal step --

def _rand_case(seed, U=2, n_cur=9, L=20, d=16):
    rng = np.random.default_rng(seed)
    q, kc, vc = (rng.standard_normal((U, n_cur, d)) for _ in range(3))
    ks, vs = rng.standard_normal((U, L, d)), rng.standard_normal((U, L, d))
    return q, kc, vc, ks, vs


def test_literal_step_attention_is_library_attention_over_history_and_current_for_any_budget():
    q, kc, vc, ks, vs = _rand_case(20)
    want = _sdpa(q, np.concatenate([ks, kc], 1), np.concatenate([vs, vc], 1))
    for budget in (0, 3, 100):
        r = oracle.step_append_first(q, kc, vc, [2, 7], ks, vs, budget)
        np.testing.assert_allclose(r["out"], want, atol=1e-12)


def test_literal_step_full_budget_keeps_everything_in_order_and_agrees_with_the_other_order():
    q, kc, vc, ks, vs = _rand_case(21)
    r = oracle.step_append_first(q, kc, vc, [0, 8], ks, vs, 10 ** 6)
    assert r["keep"] == 29 and r["idx"][0].tolist() == list(range(29))
    assert np.array_equal(r["k_next"], np.concatenate([ks, kc], 1))
    assert np.array_equal(r["v_next"], np.concatenate([vs, vc], 1))
    # with nothing evicted both orders of the step are plain attention over the same keys
    np.testing.assert_allclose(r["out"], oracle.step(q, kc, vc, [0, 8], ks, vs, 10 ** 6)["out"], atol=1e-12)


def test_literal_step_scores_are_normalised_over_history_and_current_map():
    q, kc, vc, ks, vs = _rand_case(22)
    win = [1, 4, 6]
    r = oracle.step_append_first(q, kc, vc, win, ks, vs, 5)
    # Eq. 5 with the softmax over all 29 keys: every window row sums to 1, so the scores sum to |W|
    np.testing.assert_allclose(r["scores"].sum(1), len(win), rtol=1e-12)
    # and they are the column sums of library softmax rows
    k_all = np.concatenate([ks, kc], 1)
    logits = torch.from_numpy(np.einsum("ujc,uic->uji", q[:, win], k_all) / 4.0)
    want = torch.softmax(logits, -1).sum(1).numpy()
    np.testing.assert_allclose(r["scores"], want, rtol=1e-10)


def test_literal_step_keeps_window_plus_budget_and_gathers_both_tensors():
    q, kc, vc, ks, vs = _rand_case(23)
    win = [0, 5]
    L, n_cur = 20, 9
    for budget in (0, 1, 6, 27, 28):
        r = oracle.step_append_first(q, kc, vc, win, ks, vs, budget)
        assert r["keep"] == len(win) + min(budget, L + n_cur - len(win))
        idx = r["idx"][0]
        assert L + 0 in idx and L + 5 in idx                       # window tokens preserved
        k_all, v_all = np.concatenate([ks, kc], 1), np.concatenate([vs, vc], 1)
        assert np.array_equal(r["k_next"][0], k_all[0, idx])
        assert np.array_equal(r["v_next"][0], v_all[0, idx])
        # the non-window part is the plain top-budget of the non-window scores
        rest = np.array([i for i in range(L + n_cur) if i not in (L, L + 5)])
        top = rest[oracle.select(r["scores"][:1, rest], budget)[0]]
        assert sorted(set(idx.tolist()) - {L, L + 5}) == sorted(top.tolist())


def test_literal_step_one_hot_window_points_at_one_history_key():
    rng = np.random.default_rng(24)
    n_cur, L, d = 8, 30, 16
    ks = rng.standard_normal((1, L, d)) * 0.1
    vs = rng.standard_normal((1, L, d))
    q = rng.standard_normal((1, n_cur, d)) * 0.1
    kc, vc = rng.standard_normal((1, n_cur, d)) * 0.1, rng.standard_normal((1, n_cur, d))
    direction = rng.standard_normal(d); direction /= np.linalg.norm(direction)
    win = [2, 6]
    q[0, win] = 5.0 * direction
    ks[0, 17] = 40.0 * direction
    r = oracle.step_append_first(q, kc, vc, win, ks, vs, 1)
    assert r["idx"][0].tolist() == [17, L + 2, L + 6]


def test_literal_step_pooling_spreads_a_spike_to_its_neighbours():
    rng = np.random.default_rng(25)
    n_cur, L, d = 4, 24, 8
    ks = np.zeros((1, L, d)); vs = rng.standard_normal((1, L, d))
    kc = np.zeros((1, n_cur, d)); vc = rng.standard_normal((1, n_cur, d))
    q = np.zeros((1, n_cur, d))
    e0 = np.zeros(d); e0[0] = 1.0
    q[0, 3] = 10.0 * e0
    ks[0, 11] = 10.0 * e0                 # one spike at history position 11, everything else flat
    no_pool = oracle.step_append_first(q, kc, vc, [3], ks, vs, 3, pool_w=1)
    pooled = oracle.step_append_first(q, kc, vc, [3], ks, vs, 3, pool_w=3)
    # without pooling the spike is kept and the other two slots fall to the lowest indices (ties)
    assert no_pool["idx"][0].tolist() == [0, 1, 11, L + 3]
    # with width 3 the spike's neighbours outrank the flat rest
    assert pooled["idx"][0].tolist() == [10, 11, 12, L + 3]
    np.testing.assert_allclose(pooled["scores"], oracle.pool(no_pool["scores"], 3), rtol=1e-15)


def test_literal_step_forced_indices_are_followed():
    q, kc, vc, ks, vs = _rand_case(26)
    forced = np.array([[1, 2, 25], [0, 3, 28]], dtype=np.int32)
    r = oracle.step_append_first(q, kc, vc, [4], ks, vs, 2, force_idx=forced)
    assert np.array_equal(r["idx"], forced)
    assert np.array_equal(r["k_next"][1], np.concatenate([ks, kc], 1)[1, [0, 3, 28]])
