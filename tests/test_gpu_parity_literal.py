"""GPU parity for the literal order of Sec. 3.3 (append -> attend -> score over
history and current map -> pool -> keep window + top-budget -> compact), through
the C ABI against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_19602_amd as skv
import workloads as W
from parity_util import check_indices, check_output, units

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _rand(key, shape, dtype, scale=1.0):
    return (W.normal_tensor(W.stream_key(4321, key), shape) * scale).to(dtype)


def _note(msg):
    print(msg, flush=True)


def check_window_indices(gpu_idx, scores, forced, budget, oracle_idx):
    """Index rule with preserved positions: they must all be present; what remains is
    judged like a plain top-k over the other tokens (exact when the margin is wide,
    a valid choice inside the near-tie band otherwise)."""
    gpu_idx, oracle_idx = np.asarray(gpu_idx), np.asarray(oracle_idx)
    n = len(scores)
    forced = sorted(int(f) for f in forced)
    assert gpu_idx.shape == oracle_idx.shape
    assert np.all(np.diff(gpu_idx) > 0)
    assert set(forced) <= set(gpu_idx.tolist()), "a window token was dropped"
    rest = np.array([i for i in range(n) if i not in set(forced)], dtype=np.int64)
    pick = min(budget, len(rest))
    to_rank = lambda idx: np.searchsorted(rest, np.array([i for i in idx.tolist() if i not in set(forced)], dtype=np.int64))
    return check_indices(to_rank(gpu_idx), scores[rest], pick, to_rank(oracle_idx))


# ------------------------------------------------- selection with a window --

@pytest.mark.parametrize("L,budget,n_forced,pool_w,kind", [
    (1000, 100, 16, 1, "normal"), (1000, 100, 0, 5, "normal"), (1000, 100, 16, 5, "normal"),
    (777, 300, 7, 1, "ties"), (777, 300, 7, 3, "ties"), (64, 10, 3, 7, "equal"), (64, 0, 5, 1, "normal"),
    (300, 290, 16, 3, "normal"), (300, 1000, 4, 3, "normal"), (5, 2, 1, 31, "normal"),
    (6489, 649, 16, 13, "normal"), (13000, 650, 16, 1, "normal"), (13000, 650, 16, 5, "normal"),
])
def test_select_window_matches_oracle(L, budget, n_forced, pool_w, kind):
    S, H = 2, 3
    _note(f"select_window L={L} budget={budget} n_forced={n_forced} pool_w={pool_w} kind={kind}")
    shape = skv.Shape(S, H, 128, torch.bfloat16)
    g = torch.Generator().manual_seed(L * 31 + budget)
    if kind == "normal":
        ls = torch.randn(S, H, L, generator=g) * 3.0
    elif kind == "ties":
        ls = torch.randint(0, 6, (S, H, L), generator=g).float() * 0.5 - 2.0
    else:
        ls = torch.full((S, H, L), -1.25)
    forced = sorted(torch.randperm(L, generator=g)[:n_forced].tolist())
    keep = n_forced + max(0, min(budget, L - n_forced))
    idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
    got_keep = skv.select_window(shape, ls.to(DEV), L, budget, forced, pool_w, idx)
    torch.cuda.synchronize()
    assert got_keep == keep
    pooled = oracle.pool_log(ls.double().numpy().reshape(S * H, L), pool_w)   # log of the pooled scores
    want = oracle.select_forced(pooled, budget, forced)
    got = idx.cpu().numpy().reshape(S * H, keep)
    for u in range(S * H):
        if pool_w == 1:
            assert np.array_equal(got[u], want[u])                # integer compares only: exact, ties included
        else:
            check_window_indices(got[u], pooled[u], forced, budget, want[u])


# ------------------------------------------------------------ the literal step --

def _run_literal_chain(cfg, layers, unit_ids, check_all_units, pool_w, last_scale=None, keep_all_before_first=False):
    """keep_all_before_first: scales before the first compressed one keep the map as well (the
    budget rule of the bench's literal variant); otherwise the table's budget is used as it is."""
    dtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    S, H, d = cfg.n_seq, cfg.n_head, cfg.head_dim
    shape = skv.Shape(S, H, d, dtype)
    K = last_scale or cfg.n_scale
    cap = cfg.prefix + sum(cfg.n_tokens(k) for k in range(1, K + 1))
    table = W.budget_table(cfg)
    ws = torch.empty(skv.workspace_bytes(shape, cap, max(cfg.n_tokens(k) for k in range(1, K + 1))),
                     dtype=torch.uint8, device=DEV)
    stats = dict(exact=0, band=0, max_err=0.0, moved=0)
    for layer in layers:
        kp, vp = W.make_prefix(cfg, layer, DEV)
        bufs = [(torch.zeros(S, H, cap, d, dtype=dtype, device=DEV), torch.zeros(S, H, cap, d, dtype=dtype, device=DEV))
                for _ in range(2)]
        cur = 0
        bufs[0][0][:, :, :cfg.prefix] = kp
        bufs[0][1][:, :, :cfg.prefix] = vp
        cache_len = cfg.prefix
        u_sel = list(range(S * H)) if check_all_units else unit_ids
        ref_k = units(kp)[u_sel].double().numpy(); ref_v = units(vp)[u_sel].double().numpy()
        for k in range(1, K + 1):
            side = cfg.sides[k - 1]
            n_cur, budget = cfg.n_tokens(k), table[layer][k - 1]
            if keep_all_before_first and k < cfg.first_compressed_scale:
                budget = W.c_full(cfg, k) + n_cur
            win = skv.window_centroids(side, side, 4, 4)
            assert win == oracle.window_centroids(side, side, 4, 4).tolist()
            _note(f"literal step cfg={cfg.name} layer={layer} scale={k} cache_len={cache_len} budget={budget} "
                  f"n_win={len(win)} pool_w={pool_w}")
            x = W.make_step_inputs(cfg, layer, k, DEV)
            total = cache_len + n_cur
            keep = len(win) + min(budget, total - len(win))
            k_cache, v_cache = bufs[cur]
            k_next, v_next = bufs[1 - cur]
            out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
            idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
            got_keep, moved = skv.step_append_first(shape, x.q, x.k_cur, x.v_cur, win, pool_w, k_cache, v_cache,
                                                    cache_len, budget, k_next, v_next, out, idx, ws)
            torch.cuda.synchronize()
            assert got_keep == keep and moved == (keep < total)
            g_idx = idx.cpu().numpy().reshape(S * H, keep)[u_sel]
            q_u, kc_u, vc_u = (units(t)[u_sel] for t in (x.q, x.k_cur, x.v_cur))
            # the oracle's own choice from its score, pooling and selection stages (the attention, the
            # expensive part, is computed once, below, on the choice that is followed)
            forced = [cache_len + w for w in win]
            _, own_ls = oracle.score(q_u[:, win], np.concatenate([ref_k, kc_u.double().numpy()], 1))
            own_ls = oracle.pool_log(own_ls, pool_w)
            own_idx = oracle.select_forced(own_ls, budget, forced)
            assert own_idx.shape[1] == keep
            for i in range(len(u_sel)):
                stats[check_window_indices(g_idx[i], own_ls[i], forced, budget, own_idx[i])] += 1
            ref = oracle.step_append_first(q_u, kc_u, vc_u, win, ref_k, ref_v, budget, pool_w=pool_w, force_idx=g_idx)
            # the appended rows are in place, bit-exact, whether or not anything was dropped
            assert np.array_equal(units(k_cache)[u_sel, cache_len:total].double().numpy(), kc_u.double().numpy())
            assert np.array_equal(units(v_cache)[u_sel, cache_len:total].double().numpy(), vc_u.double().numpy())
            held_k, held_v = (k_next, v_next) if moved else (k_cache, v_cache)
            assert np.array_equal(units(held_k)[u_sel, :keep].double().numpy(), ref["k_next"])
            assert np.array_equal(units(held_v)[u_sel, :keep].double().numpy(), ref["v_next"])
            mx, _ = check_output(units(out)[u_sel], ref["out"], dtype, f"literal step l{layer} k{k}")
            stats["max_err"] = max(stats["max_err"], mx)
            stats["moved"] += int(moved)
            ref_k, ref_v = ref["k_next"], ref["v_next"]
            cache_len = keep
            if moved:
                cur = 1 - cur
    return stats


@pytest.mark.parametrize("pool_w", [1, 3])
def test_literal_chain_tiny_fp32_all_units(pool_w):
    cfg = W.get_config("tiny")
    stats = _run_literal_chain(cfg, range(cfg.n_layer), None, True, pool_w)
    _note(f"literal tiny pool_w={pool_w}: {stats}")
    assert stats["exact"] + stats["band"] == cfg.n_layer * cfg.n_scale * cfg.n_seq * cfg.n_head
    assert stats["moved"] > 0


@pytest.mark.parametrize("pool_w", [1, 5])
def test_literal_chain_2b_512_sampled_units(pool_w):
    cfg = W.get_config("2b_512")
    stats = _run_literal_chain(cfg, [0, 17], [0, 5, 15], False, pool_w)
    _note(f"literal 2b_512 pool_w={pool_w}: {stats}")
    assert stats["exact"] > 0 and stats["moved"] >= 14


def test_literal_chain_2b_1024_full_size_sampled_units():
    """The literal order at the size and in the configuration `bench.py --variant literal` times:
    workload 2b_1024 on all 256 units, all 13 scales of one layer, 4x4 patch-centroid window, pooling
    width 7, nothing dropped before the first compressed scale; two units followed by the oracle."""
    cfg = W.get_config("2b_1024")
    stats = _run_literal_chain(cfg, [5], [3, 200], False, 7, keep_all_before_first=True)
    _note(f"literal 2b_1024 pool_w=7: {stats}")
    assert stats["exact"] + stats["band"] == cfg.n_scale * 2
    assert stats["moved"] == cfg.n_scale - cfg.first_compressed_scale + 1


def test_literal_step_edge_cases():
    dtype, d, S, H = torch.bfloat16, 128, 1, 2
    shape = skv.Shape(S, H, d, dtype)
    L, n_cur = 200, 36
    q, kc, vc = (_rand(70 + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
    ks, vs = _rand(73, (S, H, L, d), dtype), _rand(74, (S, H, L, d), dtype)
    cap = L + n_cur
    ws = torch.empty(skv.workspace_bytes(shape, cap, n_cur), dtype=torch.uint8, device=DEV)
    win = skv.window_centroids(6, 6)
    assert len(win) == 16

    def fresh():
        kcache = torch.zeros(S, H, cap, d, dtype=dtype, device=DEV); vcache = torch.zeros_like(kcache)
        kcache[:, :, :L] = ks.to(DEV); vcache[:, :, :L] = vs.to(DEV)
        return kcache, vcache

    # budget 0: only the window survives
    _note("literal edge: budget 0")
    kcache, vcache = fresh()
    kn = torch.zeros(S, H, cap, d, dtype=dtype, device=DEV); vn = torch.zeros_like(kn)
    out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
    idx = torch.full((S, H, 16), -1, dtype=torch.int32, device=DEV)
    keep, moved = skv.step_append_first(shape, q, kc, vc, win, 1, kcache, vcache, L, 0, kn, vn, out, idx, ws)
    torch.cuda.synchronize()
    assert (keep, moved) == (16, True)
    assert idx.cpu()[0, 0].tolist() == [L + w for w in win] and idx.cpu()[0, 1].tolist() == [L + w for w in win]
    assert torch.equal(kn[:, :, :16], kc[:, :, win]) and torch.equal(vn[:, :, :16], vc[:, :, win])
    ref = oracle.step_append_first(units(q), units(kc), units(vc), win, units(ks), units(vs), 0)
    check_output(units(out), ref["out"], dtype, "literal budget 0")

    # nothing dropped: the cache stays in place, next buffers may be absent, indices are the identity
    for budget in (L + n_cur - 16, 10 ** 6):
        _note(f"literal edge: budget {budget} keeps everything")
        kcache, vcache = fresh()
        idx = torch.full((S, H, cap), -1, dtype=torch.int32, device=DEV)
        keep, moved = skv.step_append_first(shape, q, kc, vc, win, 3, kcache, vcache, L, budget, None, None, out,
                                            idx, None)
        torch.cuda.synchronize()
        assert (keep, moved) == (cap, False)
        assert torch.equal(idx.cpu()[0, 1], torch.arange(cap, dtype=torch.int32))
        assert torch.equal(kcache[:, :, L:], kc) and torch.equal(vcache[:, :, :L], vs.to(DEV))
        check_output(units(out), ref["out"], dtype, "literal keep-all")   # attention does not depend on the budget

    # no window at all is legal as long as nothing has to be ranked
    _note("literal edge: empty window, keep everything")
    kcache, vcache = fresh()
    keep, moved = skv.step_append_first(shape, q, kc, vc, [], 1, kcache, vcache, L, 10 ** 6, None, None, out, None, None)
    torch.cuda.synchronize()
    assert (keep, moved) == (cap, False)
    with pytest.raises(skv.ScaleKVError):
        skv.step_append_first(shape, q, kc, vc, [], 1, kcache, vcache, L, 5, kn, vn, out, None, ws)


def test_literal_step_long_cache_uses_the_two_kernel_route():
    # more keys than the fused select holds in LDS: finalise + select from global, with window and pooling
    dtype, d, S, H = torch.bfloat16, 128, 1, 2
    shape = skv.Shape(S, H, d, dtype)
    L, n_cur, budget, pool_w = 12990, 64, 500, 3
    _note(f"literal long cache L={L}")
    q, kc, vc = (_rand(80 + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
    ks, vs = _rand(83, (S, H, L, d), dtype), _rand(84, (S, H, L, d), dtype)
    cap = L + n_cur
    kcache = torch.zeros(S, H, cap, d, dtype=dtype, device=DEV); vcache = torch.zeros_like(kcache)
    kcache[:, :, :L] = ks.to(DEV); vcache[:, :, :L] = vs.to(DEV)
    win = skv.window_centroids(8, 8)
    keep = 16 + budget
    kn = torch.zeros(S, H, keep, d, dtype=dtype, device=DEV); vn = torch.zeros_like(kn)
    out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
    idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(skv.workspace_bytes(shape, cap, n_cur), dtype=torch.uint8, device=DEV)
    got_keep, moved = skv.step_append_first(shape, q, kc, vc, win, pool_w, kcache, vcache, L, budget, kn, vn, out, idx, ws)
    torch.cuda.synchronize()
    assert (got_keep, moved) == (keep, True)
    own = oracle.step_append_first(units(q), units(kc), units(vc), win, units(ks), units(vs), budget, pool_w=pool_w)
    g_idx = idx.cpu().numpy().reshape(S * H, keep)
    for u in range(S * H):
        check_window_indices(g_idx[u], own["log_scores"][u], [L + w for w in win], budget, own["idx"][u])
    ref = oracle.step_append_first(units(q), units(kc), units(vc), win, units(ks), units(vs), budget, pool_w=pool_w,
                                   force_idx=g_idx)
    assert np.array_equal(units(kn).double().numpy(), ref["k_next"])
    assert np.array_equal(units(vn).double().numpy(), ref["v_next"])
    check_output(units(out), ref["out"], dtype, "literal long cache")


def test_literal_step_sweep_of_sizes_around_the_tile_edges():
    """Seeded sweep of whole literal-order steps whose map and cache sizes sit on and next to the
    kernels' tile edges, with scattered windows, pooling widths 1..7 and both dtypes / head sizes;
    every unit is followed by the oracle."""
    rng = np.random.default_rng(20250520)
    edges_q = [1, 2, 31, 32, 33, 64, 65, 127, 128, 129, 160, 161, 255, 256, 257]
    edges_l = [0, 1, 16, 17, 63, 64, 65, 128, 129, 255, 256, 257, 500]
    for case in range(24):
        dtype = torch.bfloat16 if case % 3 else torch.float32
        d = 128 if case % 2 else 64
        S, H = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        n_cur, L = int(rng.choice(edges_q)), int(rng.choice(edges_l))
        total = L + n_cur
        n_win = int(rng.integers(1, min(16, n_cur) + 1))
        win = sorted(int(x) for x in rng.choice(n_cur, size=n_win, replace=False))
        budget = int(rng.choice([0, 1, max(1, total // 4), max(0, total - n_win - 1), total - n_win, total + 3]))
        pool_w = int(rng.choice([1, 3, 5, 7]))
        keep = n_win + min(budget, total - n_win)
        _note(f"literal sweep case={case} dtype={dtype} d={d} S={S} H={H} n_cur={n_cur} L={L} budget={budget} "
              f"n_win={n_win} pool_w={pool_w}")
        shape = skv.Shape(S, H, d, dtype)
        q, kc, vc = (_rand(1500 + 7 * case + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
        ks, vs = (_rand(1500 + 7 * case + 3 + i, (S, H, max(L, 1), d), dtype)[:, :, :L] for i in range(2))
        k_cache = torch.zeros(S, H, total, d, dtype=dtype, device=DEV); v_cache = torch.zeros_like(k_cache)
        k_cache[:, :, :L] = ks.to(DEV); v_cache[:, :, :L] = vs.to(DEV)
        k_next = torch.zeros(S, H, total, d, dtype=dtype, device=DEV); v_next = torch.zeros_like(k_next)
        ws = torch.empty(skv.workspace_bytes(shape, total, n_cur), dtype=torch.uint8, device=DEV)
        out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        got_keep, moved = skv.step_append_first(shape, q, kc, vc, win, pool_w, k_cache, v_cache, L, budget,
                                                k_next, v_next, out, idx, ws)
        torch.cuda.synchronize()
        assert got_keep == keep and moved == (keep < total)
        g_idx = idx.cpu().numpy().reshape(S * H, keep)
        own = oracle.step_append_first(units(q), units(kc), units(vc), win, units(ks), units(vs), budget, pool_w=pool_w)
        assert own["keep"] == keep
        forced = [L + w for w in win]
        for u in range(S * H):
            check_window_indices(g_idx[u], own["log_scores"][u], forced, budget, own["idx"][u])
        ref = oracle.step_append_first(units(q), units(kc), units(vc), win, units(ks), units(vs), budget,
                                       pool_w=pool_w, force_idx=g_idx)
        assert torch.equal(k_cache[:, :, L:], kc) and torch.equal(v_cache[:, :, L:], vc)
        held_k, held_v = (k_next, v_next) if moved else (k_cache, v_cache)
        assert np.array_equal(units(held_k)[:, :keep].double().numpy(), ref["k_next"])
        assert np.array_equal(units(held_v)[:, :keep].double().numpy(), ref["v_next"])
        check_output(units(out), ref["out"], dtype, f"literal sweep case {case}")
