"""Pins for the fp64 oracle: closed forms, invariants, library routines and the
numbers the paper prints.  None of these retype the oracle's own loops; each
would fail for a plausible slip (dropped term, sign, index, transposed operand,
sum-vs-mean, wrong tie-break)."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _paper_numbers():
    out = {}
    for line in open(os.path.join(GOLD, "paper_numbers.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


# ------------------------------------------------------------------ score --

def test_score_rows_are_distributions_and_sum_is_window_size():
    rng = np.random.default_rng(1)
    qw = rng.standard_normal((3, 5, 24)) * 2
    k = rng.standard_normal((3, 37, 24)) * 2
    s, ls, a = oracle.score(qw, k, return_attention=True)
    assert np.all(a >= 0)
    np.testing.assert_allclose(a.sum(-1), 1.0, rtol=0, atol=1e-13)
    # Eq. 5 sums (does not average) over the window, so the scores total N.
    np.testing.assert_allclose(s.sum(-1), 5.0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(s, a.sum(1), rtol=0, atol=1e-14)
    np.testing.assert_allclose(ls, np.log(s), rtol=0, atol=1e-12)


def test_score_identical_keys_give_uniform_scores():
    rng = np.random.default_rng(2)
    qw = rng.standard_normal((1, 7, 16))
    k = np.tile(rng.standard_normal((1, 1, 16)), (1, 29, 1))
    s, ls = oracle.score(qw, k)
    np.testing.assert_allclose(s, 7.0 / 29.0, rtol=1e-13)
    np.testing.assert_allclose(ls, math.log(7.0 / 29.0), rtol=0, atol=1e-13)


def test_score_closed_form_orthogonal_keys():
    # keys are c * e_i (i < len <= d); window query j is a_j * e_{p_j}: the only
    # non-zero logit of row j sits at key p_j and equals a_j * c / sqrt(d).
    d, length = 12, 9
    c = 1.7
    a = np.array([0.5, 3.0, -2.0, 8.0])
    p = np.array([4, 0, 4, 7])
    k = np.zeros((1, length, d)); k[0, np.arange(length), np.arange(length)] = c
    qw = np.zeros((1, len(a), d)); qw[0, np.arange(len(a)), p] = a
    s, ls, att = oracle.score(qw, k, return_attention=True)
    expect = np.zeros(length)
    for aj, pj in zip(a, p):
        x = aj * c / math.sqrt(d)
        z = math.exp(x) + (length - 1)
        row = np.full(length, 1.0 / z); row[pj] = math.exp(x) / z
        expect += row
    np.testing.assert_allclose(s[0], expect, rtol=1e-13)
    # explicit scale overrides 1/sqrt(d)
    s2, _ = oracle.score(qw, k, scale=0.25)
    expect2 = np.zeros(length)
    for aj, pj in zip(a, p):
        x = aj * c * 0.25
        z = math.exp(x) + (length - 1)
        row = np.full(length, 1.0 / z); row[pj] = math.exp(x) / z
        expect2 += row
    np.testing.assert_allclose(s2[0], expect2, rtol=1e-13)


def test_score_single_window_row_is_library_softmax():
    rng = np.random.default_rng(3)
    qw = rng.standard_normal((2, 1, 40))
    k = rng.standard_normal((2, 23, 40))
    s, _ = oracle.score(qw, k)
    for u in range(2):
        lib = scipy.special.softmax(k[u] @ qw[u, 0] / math.sqrt(40))
        np.testing.assert_allclose(s[u], lib, rtol=1e-12)


def test_score_many_rows_against_library_softmax():
    rng = np.random.default_rng(4)
    qw = rng.standard_normal((1, 6, 20)) * 3
    k = rng.standard_normal((1, 50, 20)) * 3
    s, _ = oracle.score(qw, k)
    lib = torch.softmax(torch.from_numpy(qw[0] @ k[0].T) / math.sqrt(20), dim=-1).sum(0).numpy()
    np.testing.assert_allclose(s[0], lib, rtol=1e-12)


def test_log_score_survives_underflow():
    # one enormous logit per row: every other probability underflows in exp()
    # but its log stays finite and ordered.
    d = 4
    k = np.zeros((1, 6, d)); k[0, :, 0] = [0, 1, 2, 3, 4, 2000]
    qw = np.zeros((1, 2, d)); qw[0, :, 0] = [2.0, 2.0]
    s, ls = oracle.score(qw, k, scale=1.0)
    assert s[0, 0] == 0.0 and s[0, 5] == pytest.approx(2.0)
    assert np.all(np.isfinite(ls[0]))
    assert np.all(np.diff(ls[0]) > 0)
    np.testing.assert_allclose(ls[0, :5], 2.0 * np.arange(5) - 4000.0 + math.log(2.0), rtol=1e-12)


# ----------------------------------------------------------------- select --

def _brute(scores, budget):
    order = sorted(range(len(scores)), key=lambda i: (-scores[i], i))
    return sorted(order[: min(budget, len(scores))])


def test_select_matches_full_sort_on_tiny_inputs():
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(1, 65))
        # few distinct values => many exact ties
        s = rng.integers(0, 6, size=n).astype(np.float64) / 8.0
        b = int(rng.integers(0, n + 4))
        got = oracle.select(s[None], b)[0].tolist()
        assert got == _brute(s.tolist(), b), (trial, n, b)


def test_select_all_equal_takes_lowest_indices():
    s = np.full((1, 40), 0.125)
    assert oracle.select(s, 7)[0].tolist() == list(range(7))


def test_select_budget_edge_cases_and_nesting():
    rng = np.random.default_rng(6)
    s = rng.random((2, 33))
    assert oracle.select(s, 0).shape == (2, 0)
    assert oracle.select(s, 33)[1].tolist() == list(range(33))
    assert oracle.select(s, 1000)[0].tolist() == list(range(33))
    small, big = oracle.select(s, 5), oracle.select(s, 12)
    for u in range(2):
        assert set(small[u]) < set(big[u])
        assert small[u].tolist() == sorted(small[u].tolist())
        assert int(np.argmax(s[u])) in small[u]


# ---------------------------------------------------------------- compact --

def test_compact_rows_and_append():
    rng = np.random.default_rng(7)
    src = rng.standard_normal((2, 11, 6)); cur = rng.standard_normal((2, 3, 6))
    idx = np.array([[0, 4, 9, 10], [2, 3, 5, 7]], dtype=np.int32)
    dst = oracle.compact(src, idx, cur)
    assert dst.shape == (2, 7, 6)
    for u in range(2):
        for t in range(4):
            assert np.array_equal(dst[u, t], src[u, idx[u, t]])
        assert np.array_equal(dst[u, 4:], cur[u])
    ident = np.tile(np.arange(11, dtype=np.int32), (2, 1))
    assert np.array_equal(oracle.compact(src, ident, cur)[:, :11], src)


# ----------------------------------------------------------------- attend --

def _sdpa(q, k, v, scale=None):
    q, k, v = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (q, k, v))
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=scale).numpy()


def test_attend_equals_library_attention():
    rng = np.random.default_rng(8)
    q = rng.standard_normal((3, 13, 32)) * 2
    k = rng.standard_normal((3, 45, 32)) * 2
    v = rng.standard_normal((3, 45, 32))
    np.testing.assert_allclose(oracle.attend(q, k, v), _sdpa(q, k, v), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.attend(q, k, v, scale=0.3), _sdpa(q, k, v, scale=0.3), rtol=0, atol=1e-12)


def test_attend_special_cases():
    rng = np.random.default_rng(9)
    q = rng.standard_normal((1, 5, 16)); k = rng.standard_normal((1, 21, 16)); v = rng.standard_normal((1, 21, 16))
    vv = np.tile(rng.standard_normal((1, 1, 16)), (1, 21, 1))
    np.testing.assert_allclose(oracle.attend(q, k, vv), np.tile(vv[:, :1], (1, 5, 1)), atol=1e-13)
    np.testing.assert_allclose(oracle.attend(np.zeros_like(q), k, v),
                               np.tile(v.mean(1, keepdims=True), (1, 5, 1)), atol=1e-13)
    perm = rng.permutation(21)
    np.testing.assert_allclose(oracle.attend(q, k[:, perm], v[:, perm]), oracle.attend(q, k, v), atol=1e-13)
    np.testing.assert_allclose(oracle.attend(q, k[:, :1], v[:, :1]), np.tile(v[:, :1], (1, 5, 1)), atol=0)


# ------------------------------------------------------------------- step --

def test_step_with_full_budget_is_plain_attention_over_cache_and_current():
    rng = np.random.default_rng(10)
    U, n_cur, L, d = 2, 9, 30, 16
    q, kc, vc = (rng.standard_normal((U, n_cur, d)) for _ in range(3))
    ks, vs = rng.standard_normal((U, L, d)), rng.standard_normal((U, L, d))
    for budget in (L, L + 5):
        r = oracle.step(q, kc, vc, [7, 8], ks, vs, budget)
        assert r["new_len"] == L + n_cur
        assert np.array_equal(r["k_dst"], np.concatenate([ks, kc], 1))
        assert np.array_equal(r["v_dst"], np.concatenate([vs, vc], 1))
        np.testing.assert_allclose(r["out"], _sdpa(q, np.concatenate([ks, kc], 1), np.concatenate([vs, vc], 1)),
                                   atol=1e-12)


def test_step_budget_zero_attends_over_current_only():
    rng = np.random.default_rng(11)
    q, kc, vc = (rng.standard_normal((1, 6, 8)) for _ in range(3))
    ks, vs = rng.standard_normal((1, 10, 8)), rng.standard_normal((1, 10, 8))
    r = oracle.step(q, kc, vc, [5], ks, vs, 0)
    assert r["new_len"] == 6 and r["idx"].shape == (1, 0)
    np.testing.assert_allclose(r["out"], _sdpa(q, kc, vc), atol=1e-12)


def test_step_one_hot_pattern_selects_its_argmax_and_uses_window_rows():
    rng = np.random.default_rng(12)
    n_cur, L, d = 12, 40, 16
    ks = rng.standard_normal((1, L, d)) * 0.1
    vs = rng.standard_normal((1, L, d))
    q = rng.standard_normal((1, n_cur, d)) * 0.1
    kc, vc = rng.standard_normal((1, n_cur, d)), rng.standard_normal((1, n_cur, d))
    win = [3, 10]
    direction = rng.standard_normal(d); direction /= np.linalg.norm(direction)
    q[0, win] = 5.0 * direction          # only the window rows point at the target
    ks[0, 23] = 40.0 * direction         # the target key
    for budget in (1, 2, 9):
        r = oracle.step(q, kc, vc, win, ks, vs, budget)
        assert 23 in r["idx"][0]
        assert r["idx"].shape == (1, budget)
    # the scores really come from rows `win` of q, nobody else
    s, _ = oracle.score(q[:, win], ks)
    assert np.array_equal(oracle.step(q, kc, vc, win, ks, vs, 3)["scores"], s)
    # and the kept rows are gathered from both K and V with the same indices
    r = oracle.step(q, kc, vc, win, ks, vs, 4)
    assert np.array_equal(r["k_dst"][0, :4], ks[0, r["idx"][0]])
    assert np.array_equal(r["v_dst"][0, :4], vs[0, r["idx"][0]])
    np.testing.assert_allclose(r["out"], _sdpa(q, r["k_dst"], r["v_dst"]), atol=1e-12)


def test_step_ranks_on_log_scores_same_choice_where_nothing_underflows():
    # Sec. 3.3's top-k depends only on the order of the scores; log is strictly increasing, so the
    # step (which ranks log s) must choose what a ranking of s itself chooses.  Independent check:
    # the linear scores come from a library softmax, the choice from a full sort.
    rng = np.random.default_rng(41)
    for trial in range(20):
        n_cur, L, d, budget = 6, int(rng.integers(8, 60)), 12, int(rng.integers(1, 8))
        q, kc, vc = (rng.standard_normal((2, n_cur, d)) * 2 for _ in range(3))
        ks, vs = rng.standard_normal((2, L, d)) * 2, rng.standard_normal((2, L, d))
        win = [1, 4, 5]
        r = oracle.step(q, kc, vc, win, ks, vs, budget)
        for u in range(2):
            lib = torch.softmax(torch.from_numpy(q[u][win] @ ks[u].T) / math.sqrt(d), dim=-1).sum(0).numpy()
            assert lib.min() > 1e-200                                     # nothing underflows here
            assert r["idx"][u].tolist() == _brute(lib.tolist(), budget), trial
            np.testing.assert_allclose(r["log_scores"][u], np.log(lib), rtol=0, atol=1e-11)
        assert np.array_equal(oracle.select(r["scores"], budget), oracle.select(r["log_scores"], budget))


def test_step_still_ranks_where_the_scores_underflow():
    # One window row and logits thousands apart: every score but the largest is 0.0 in fp64, and a
    # ranking of s would fall back on the index order.  With one row log s_i = logit_i - log Z, so
    # the order Eq. 5 defines is the order of the dot products, which numpy gives independently.
    rng = np.random.default_rng(42)
    n_cur, L, d, budget = 3, 40, 8, 9
    q, kc, vc = (rng.standard_normal((1, n_cur, d)) for _ in range(3))
    ks, vs = rng.standard_normal((1, L, d)) * 2000.0, rng.standard_normal((1, L, d))
    r = oracle.step(q, kc, vc, [2], ks, vs, budget, scale=1.0)
    assert np.count_nonzero(r["scores"][0]) < budget                       # the regime is the intended one
    logits = ks[0] @ q[0, 2]
    assert r["idx"][0].tolist() == _brute(logits.tolist(), budget)
    assert np.all(np.isfinite(r["log_scores"]))


def test_step_forced_indices_are_followed():
    rng = np.random.default_rng(13)
    q, kc, vc = (rng.standard_normal((1, 4, 8)) for _ in range(3))
    ks, vs = rng.standard_normal((1, 10, 8)), rng.standard_normal((1, 10, 8))
    forced = np.array([[1, 2, 8]], dtype=np.int32)
    r = oracle.step(q, kc, vc, [0], ks, vs, 3, force_idx=forced)
    assert np.array_equal(r["idx"], forced)
    assert np.array_equal(r["k_dst"][0, :3], ks[0, [1, 2, 8]])


# ------------------------------------------------------------ cache sizes --

def test_schedule_token_totals():
    nums = _paper_numbers()
    assert W.get_config("tiny").image_tokens == 85
    assert W.get_config("2b_512").image_tokens == 2521
    assert W.get_config("2b_1024").image_tokens == 10521
    assert W.get_config("2b_1024").image_tokens > nums["tokens_1024_lower_bound"]
    assert W.get_config("2b_1024").window == nums["window_tokens"]


def test_cache_lengths_without_eviction_are_prefix_plus_earlier_maps():
    cfg = W.get_config("2b_1024")
    n_tok = [cfg.n_tokens(k) for k in range(1, cfg.n_scale + 1)]
    li, kp, final = oracle.cache_lengths(cfg.prefix, n_tok, [10 ** 9] * cfg.n_scale)
    for k in range(1, cfg.n_scale + 1):
        assert li[k - 1] == cfg.prefix + sum(s * s for s in cfg.sides[: k - 1])
        assert kp[k - 1] == li[k - 1]
    assert final == cfg.prefix + 10521


def test_tiny_workload_cache_lengths_match_hand_worked_fixture():
    cfg = W.get_config("tiny")
    table = W.budget_table(cfg)
    n_tok = [cfg.n_tokens(k) for k in range(1, cfg.n_scale + 1)]
    rows = [tuple(int(x) for x in line.split()) for line in open(os.path.join(GOLD, "tiny_cache_lengths.txt"))
            if line.strip() and not line.startswith("#")]
    for layer in range(cfg.n_layer):
        li, kp, final = oracle.cache_lengths(cfg.prefix, n_tok, table[layer])
        for (l, k, len_in, keep, len_out) in [r for r in rows if r[0] == layer]:
            assert li[k - 1] == len_in and kp[k - 1] == keep
            nxt = li[k] if k < cfg.n_scale else final
            assert nxt == len_out


def test_ten_percent_budget_unit_matches_the_papers_650_tokens():
    # Sec. 4.3: a 10 % budget on Infinity-2B is 650 tokens per head per layer.
    nums = _paper_numbers()
    cfg = W.get_config("2b_1024")
    table = W.budget_table(cfg)
    last = cfg.n_scale
    mean_budget = sum(table[l][last - 1] for l in range(cfg.n_layer)) / cfg.n_layer
    assert abs(mean_budget - nums["budget_tokens_at_10pct"]) <= 2
    assert abs(0.10 * W.c_full(cfg, last) - nums["budget_tokens_at_10pct"]) <= 2
    # kept bytes are proportional to kept tokens (Table 1's MB column)
    assert nums["kv_mb_2b_10"] / nums["kv_mb_2b_full"] == pytest.approx(0.10, abs=0.005)
    assert nums["kv_mb_8b_10"] / nums["kv_mb_8b_full"] == pytest.approx(0.10, abs=0.005)
    assert nums["kv_gb_8b_bs8_10"] / nums["kv_gb_8b_bs8_full"] == pytest.approx(0.10, abs=0.005)


def test_budget_tables_keep_drafters_far_above_refiners():
    # Eq. 4: B_d(k) >> B_r(k); overall retention 10 % for the main workload.
    cfg = W.get_config("2b_1024")
    table = W.budget_table(cfg)
    for k in range(cfg.first_compressed_scale, cfg.n_scale + 1):
        roles = W.layer_roles(cfg, k)
        assert sum(roles) == cfg.n_drafter
        bd = {table[l][k - 1] for l in range(cfg.n_layer) if roles[l]}
        br = {table[l][k - 1] for l in range(cfg.n_layer) if not roles[l]}
        assert len(bd) == 1 and len(br) == 1 and min(bd) >= 4 * max(br)
    k = cfg.n_scale
    total = sum(table[l][k - 1] for l in range(cfg.n_layer))
    assert total / (cfg.n_layer * W.c_full(cfg, k)) == pytest.approx(0.10, abs=0.002)
