"""GPU parity: every stage and the whole step, through the C ABI, element by
element against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_19602_amd as skv
import workloads as W
from parity_util import TOL, check_indices, check_output, units

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _rand(key, shape, dtype, scale=1.0):
    return (W.normal_tensor(W.stream_key(1234, key), shape) * scale).to(dtype)


def _note(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------- compact --

@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("d", [64, 128])
def test_compact_is_bit_exact_and_stays_in_bounds(dtype, d):
    S, H, L, keep, n_cur, cap_src, cap_dst = 2, 3, 300, 77, 45, 320, 130
    _note(f"compact dtype={dtype} d={d}")
    shape = skv.Shape(S, H, d, dtype)
    ks, vs = _rand(1, (S, H, cap_src, d), dtype), _rand(2, (S, H, cap_src, d), dtype)
    kc, vc = _rand(3, (S, H, n_cur, d), dtype), _rand(4, (S, H, n_cur, d), dtype)
    gen = torch.Generator().manual_seed(5)
    idx = torch.stack([torch.sort(torch.randperm(L, generator=gen)[:keep])[0] for _ in range(S * H)])
    idx = idx.reshape(S, H, keep).to(torch.int32)
    canary = 7.0
    kd = torch.full((S, H, cap_dst, d), canary, dtype=dtype, device=DEV); vd = torch.full_like(kd, canary)
    new_len = skv.compact(shape, ks.to(DEV), vs.to(DEV), L, idx.to(DEV), keep, kc.to(DEV), vc.to(DEV), kd, vd)
    torch.cuda.synchronize()
    assert new_len == keep + n_cur
    for src, cur, dst in ((ks, kc, kd), (vs, vc, vd)):
        ref = oracle.compact(units(src)[:, :L].double(), idx.reshape(S * H, keep).numpy(), units(cur).double())
        got = units(dst).double().numpy()
        assert np.array_equal(got[:, :new_len], ref)
        assert np.all(got[:, new_len:] == canary)          # rows past the new length untouched


def test_compact_identity_strided_and_empty_parts():
    S, H, d, L, n_cur = 1, 4, 128, 50, 9
    dtype = torch.bfloat16
    shape = skv.Shape(S, H, d, dtype)
    # caches that are views into larger allocations (head stride > capacity * d)
    ks = _rand(10, (S, H, 100, d), dtype).to(DEV)[:, :, :64]
    vs = _rand(13, (S, H, 100, d), dtype).to(DEV)[:, :, :64]
    kd = torch.zeros(S, H, 128, d, dtype=dtype, device=DEV)[:, :, :80]
    vd = torch.zeros(S, H, 128, d, dtype=dtype, device=DEV)[:, :, :80]
    kc, vc = _rand(11, (S, H, n_cur, d), dtype).to(DEV), _rand(12, (S, H, n_cur, d), dtype).to(DEV)
    assert skv.compact(shape, ks, vs, L, None, L, kc, vc, kd, vd) == L + n_cur     # idx NULL = identity
    torch.cuda.synchronize()
    assert torch.equal(kd[:, :, :L], ks[:, :, :L]) and torch.equal(vd[:, :, L:L + n_cur], vc)
    assert torch.equal(kd[:, :, L:L + n_cur], kc) and torch.equal(vd[:, :, :L], vs[:, :, :L])
    # nothing kept, nothing appended: legal no-ops
    assert skv.compact(shape, ks, vs, L, None, 0, kc, vc, kd, vd) == n_cur
    assert skv.compact(shape, ks, vs, L, None, 5, None, None, kd, vd) == 5
    assert skv.compact(shape, ks, vs, 0, None, 0, None, None, kd, vd) == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------------ score --

@pytest.mark.parametrize("dtype,d,L,n_win", [
    (torch.bfloat16, 128, 1000, 16), (torch.bfloat16, 128, 257, 5), (torch.bfloat16, 128, 1, 16),
    (torch.bfloat16, 64, 700, 16), (torch.float32, 64, 333, 8), (torch.float32, 128, 64, 1),
    (torch.bfloat16, 128, 6489, 16),
])
def test_score_matches_oracle(dtype, d, L, n_win):
    S, H = 2, 2
    _note(f"score dtype={dtype} d={d} L={L} n_win={n_win}")
    shape = skv.Shape(S, H, d, dtype)
    qw = _rand(20, (S, H, n_win, d), dtype, 1.5)
    k = _rand(21, (S, H, L + 3, d), dtype, 1.5)
    ls = torch.full((S, H, L), float("nan"), device=DEV)
    ws = torch.empty(skv.workspace_bytes(shape, L, 16), dtype=torch.uint8, device=DEV)
    skv.score(shape, qw.to(DEV), k.to(DEV), L, ls, ws)
    torch.cuda.synchronize()
    s_ref, ls_ref = oracle.score(units(qw), units(k)[:, :L])
    got = ls.cpu().numpy().reshape(S * H, L).astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.abs(got - ls_ref).max() < 2e-4
    np.testing.assert_allclose(np.exp(got).sum(-1), n_win, rtol=1e-4)   # Eq. 5: scores total N


def test_score_survives_fp32_underflow():
    # peaked logits: most probabilities underflow in fp32, their logs must not
    S, H, d, L, n_win = 1, 2, 128, 500, 16
    shape = skv.Shape(S, H, d, torch.bfloat16)
    qw = _rand(22, (S, H, n_win, d), torch.bfloat16, 6.0)
    k = _rand(23, (S, H, L, d), torch.bfloat16, 6.0)
    ls = torch.empty(S, H, L, device=DEV)
    ws = torch.empty(skv.workspace_bytes(shape, L, 16), dtype=torch.uint8, device=DEV)
    skv.score(shape, qw.to(DEV), k.to(DEV), L, ls, ws)
    torch.cuda.synchronize()
    s_ref, ls_ref = oracle.score(units(qw), units(k))
    assert ls_ref.min() < -100                      # exp() of this is 0 in fp32
    got = ls.cpu().numpy().reshape(S * H, L).astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.abs(got - ls_ref).max() < 2e-3        # logits up to ~400: 1e-6 relative each


# ----------------------------------------------------------------- select --

@pytest.mark.parametrize("L,budget,kind", [
    (1000, 100, "normal"), (1000, 1, "normal"), (1000, 999, "normal"), (6489, 1622, "normal"),
    (777, 300, "ties"), (64, 10, "equal"), (5, 3, "ties"), (13000, 650, "normal"), (13000, 12999, "ties"),
    (300, 300, "normal"), (300, 1000, "normal"),
])
def test_select_is_bit_exact_on_given_scores(L, budget, kind):
    S, H = 2, 3
    _note(f"select L={L} budget={budget} kind={kind}")
    shape = skv.Shape(S, H, 128, torch.bfloat16)
    x = W.normal_tensor(W.stream_key(99, L, budget), (S, H, L))
    if kind == "ties":
        x = torch.round(x * 2) / 2            # a handful of distinct values, signed zeros included
        x[0, 0, ::7] = -0.0
    elif kind == "equal":
        x = torch.full_like(x, -3.25)
    keep = min(budget, L)
    idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
    assert skv.select(shape, x.to(DEV), L, budget, idx) == keep
    torch.cuda.synchronize()
    ref = oracle.select(x.reshape(S * H, L).double().numpy(), budget)   # same fp32 values, widened
    assert np.array_equal(idx.cpu().numpy().reshape(S * H, keep), ref)


# ----------------------------------------------------------------- attend --

@pytest.mark.parametrize("dtype,d,n_q,kv_len", [
    (torch.bfloat16, 128, 300, 700), (torch.bfloat16, 128, 1, 64), (torch.bfloat16, 128, 129, 65),
    (torch.bfloat16, 128, 128, 1), (torch.bfloat16, 128, 257, 1000), (torch.bfloat16, 64, 200, 333),
    (torch.float32, 64, 70, 150), (torch.float32, 128, 33, 95), (torch.float32, 64, 1, 1),
])
def test_attend_matches_oracle(dtype, d, n_q, kv_len):
    S, H = 2, 2
    _note(f"attend dtype={dtype} d={d} n_q={n_q} kv_len={kv_len}")
    shape = skv.Shape(S, H, d, dtype)
    q = _rand(30, (S, H, n_q, d), dtype, 1.3)
    k = _rand(31, (S, H, kv_len + 5, d), dtype, 1.3)
    v = _rand(32, (S, H, kv_len + 5, d), dtype)
    # rows past kv_len must be ignored even if they hold garbage
    k[:, :, kv_len:] = float("nan"); v[:, :, kv_len:] = float("nan")
    out = torch.full((S, H, n_q, d), float("nan"), dtype=dtype, device=DEV)
    skv.attend(shape, q.to(DEV), k.to(DEV), v.to(DEV), kv_len, out)
    torch.cuda.synchronize()
    ref = oracle.attend(units(q), units(k)[:, :kv_len], units(v)[:, :kv_len])
    mx, mean = check_output(out, ref, dtype, "attend")
    _note(f"  max {mx:.2e} mean {mean:.2e}")


@pytest.mark.parametrize("where", ["late_in_cache", "in_current_map", "second_tile", "some_rows_only",
                                   "large_but_unchecked", "huge_values"])
def test_attend_scores_far_above_the_first_tile(where):
    # Keys whose scores sit far above everything in the first 64 rows: exp2 of their distance to
    # the first tile's maximum leaves the range the kernel adds up unchecked (2^100; for the larger
    # gaps, fp32 altogether), so the workgroup has to fall back to the running-maximum scheme.
    # "large_but_unchecked": a gap of about 34 natural units (2^49), which the kernel adds up as it
    # is; "huge_values": the same gap with value rows of magnitude 2^100, whose weighted sums leave
    # fp32 although the weights do not, so the accumulators' own check has to trigger.
    S, H, d, n_q, len1, len2 = 1, 2, 128, 300, 400, 300
    dtype = torch.bfloat16
    _note(f"attend overflow fallback: {where}")
    shape = skv.Shape(S, H, d, dtype)
    q = _rand(40, (S, H, n_q, d), dtype)
    ks, vs = _rand(41, (S, H, len1 + len2, d), dtype, 0.05), _rand(42, (S, H, len1 + len2, d), dtype)
    row = {"late_in_cache": len1 - 3, "in_current_map": len1 + 170, "second_tile": 70, "some_rows_only": 333,
           "large_but_unchecked": 200, "huge_values": 200}[where]
    gain = {"late_in_cache": 9.0, "in_current_map": 30.0, "second_tile": 10.0, "some_rows_only": 10.0,
            "large_but_unchecked": 3.0, "huge_values": 3.0}[where]
    post = 1.0
    if where == "huge_values":
        vs = (vs.float() * 2.0 ** 100).to(dtype)
        post = 2.0 ** -100           # outputs are compared after this exact rescaling
    if where == "some_rows_only":       # only queries 5..9 see the large scores
        ks[:, :, row] = (q[:, :, 5].float() * gain).to(dtype)
        q[:, :, 6:10] = q[:, :, 5:6]
    else:                               # every query does: key = gain * mean direction of the queries
        q = (q.float() + 1.0).to(dtype)
        ks[:, :, row] = gain
    kc, vc = ks[:, :, len1:].contiguous(), vs[:, :, len1:].contiguous()
    out = torch.full((S, H, n_q, d), float("nan"), dtype=dtype, device=DEV)
    skv.attend(shape, q.to(DEV), ks.to(DEV), vs.to(DEV), len1 + len2, out)       # one segment
    torch.cuda.synchronize()
    ref = oracle.attend(units(q), units(ks), units(vs)) * post
    check_output(out.float() * post, ref, dtype, f"attend {where}")
    # the same keys as cache + current map through the step (budget = len1 keeps every cached row):
    # two key segments, and the kernel appends the map's K/V itself
    kd = torch.zeros(S, H, len1 + len2 + 2, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
    out2 = torch.full_like(out, float("nan"))
    new_len = skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), [0], ks[:, :, :len1].contiguous().to(DEV),
                       vs[:, :, :len1].contiguous().to(DEV), len1, len1, kd, vd, out2, None, None)
    torch.cuda.synchronize()
    assert new_len == len1 + len2
    assert torch.equal(kd[:, :, :new_len].cpu(), ks) and torch.equal(vd[:, :, :new_len].cpu(), vs)
    assert torch.all(kd[:, :, new_len:] == 0) and torch.all(vd[:, :, new_len:] == 0)
    check_output(out2.float() * post, ref, dtype, f"step {where}")


def test_attend_closed_forms_on_gpu():
    S, H, d, n_q, kv = 1, 2, 128, 140, 260
    dtype = torch.bfloat16
    shape = skv.Shape(S, H, d, dtype)
    q = _rand(33, (S, H, n_q, d), dtype).to(DEV)
    k = _rand(34, (S, H, kv, d), dtype).to(DEV)
    row = _rand(35, (S, H, 1, d), dtype).to(DEV)
    out = torch.empty(S, H, n_q, d, dtype=dtype, device=DEV)
    skv.attend(shape, q, k, row.expand(S, H, kv, d).contiguous(), kv, out)      # all V rows equal -> O = v
    torch.cuda.synchronize()
    assert (out.float() - row.float()).abs().max() < 2e-2
    v = _rand(36, (S, H, kv, d), dtype).to(DEV)
    skv.attend(shape, torch.zeros_like(q), k, v, kv, out)                       # Q = 0 -> mean of V
    torch.cuda.synchronize()
    assert (out.float() - v.float().mean(2, keepdim=True)).abs().max() < 2e-2


# ------------------------------------------------------------------- step --

def _run_chain(cfg, layers, unit_ids, check_all_units, last_scale=None, table=None):
    """Run all scales of `cfg` for the given layers on the GPU through
    scalekv_step and follow each (layer, unit) with the oracle.  `table`: budgets per
    [layer][scale - 1] in place of the config's own."""
    dtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    S, H, d = cfg.n_seq, cfg.n_head, cfg.head_dim
    shape = skv.Shape(S, H, d, dtype)
    if table is None:
        table = W.budget_table(cfg)
    cap = max(min(table[l][k - 1], W.c_full(cfg, k)) + cfg.n_tokens(k)
              for l in range(cfg.n_layer) for k in range(1, cfg.n_scale + 1))
    ws = torch.empty(skv.workspace_bytes(shape, cap, max(cfg.n_tokens(k) for k in range(1, cfg.n_scale + 1))),
                     dtype=torch.uint8, device=DEV)
    stats = dict(exact=0, band=0, max_err=0.0)
    for layer in layers:
        kp, vp = W.make_prefix(cfg, layer, DEV)
        bufs = [(torch.zeros(S, H, cap, d, dtype=dtype, device=DEV), torch.zeros(S, H, cap, d, dtype=dtype, device=DEV))
                for _ in range(2)]
        src_k, src_v, cache_len = kp, vp, cfg.prefix
        u_sel = list(range(S * H)) if check_all_units else unit_ids
        ref_k = units(kp)[u_sel].double().numpy(); ref_v = units(vp)[u_sel].double().numpy()
        for k in range(1, (last_scale or cfg.n_scale) + 1):
            _note(f"step cfg={cfg.name} layer={layer} scale={k} cache_len={cache_len}")
            x = W.make_step_inputs(cfg, layer, k, DEV)
            n_cur, budget = cfg.n_tokens(k), table[layer][k - 1]
            win = W.window_indices(cfg, n_cur)
            keep = min(budget, cache_len)
            dst_k, dst_v = bufs[k % 2]
            out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
            idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
            new_len = skv.step(shape, x.q, x.k_cur, x.v_cur, win, src_k, src_v, cache_len, budget,
                               dst_k, dst_v, out, idx, ws)
            torch.cuda.synchronize()
            assert new_len == keep + n_cur
            g_idx = idx.cpu().numpy().reshape(S * H, keep)[u_sel]
            q_u, kc_u, vc_u = (units(t)[u_sel] for t in (x.q, x.k_cur, x.v_cur))
            # the oracle's own choice from its score and select stages (the attention, the expensive
            # part, is then computed once, below, on the choice that is followed)
            _, own_ls = oracle.score(q_u[:, win], ref_k)
            own_idx = oracle.select(own_ls, budget)
            for i in range(len(u_sel)):
                stats[check_indices(g_idx[i], own_ls[i], keep, own_idx[i])] += 1
            # follow the GPU's (validated) choice so later scales stay comparable
            ref = oracle.step(q_u, kc_u, vc_u, win, ref_k, ref_v, budget, force_idx=g_idx)
            assert np.array_equal(units(dst_k)[u_sel, :new_len].double().numpy(), ref["k_dst"])   # bit-exact rows
            assert np.array_equal(units(dst_v)[u_sel, :new_len].double().numpy(), ref["v_dst"])
            mx, _ = check_output(units(out)[u_sel], ref["out"], dtype, f"step l{layer} k{k}")
            stats["max_err"] = max(stats["max_err"], mx)
            ref_k, ref_v = ref["k_dst"], ref["v_dst"]
            src_k, src_v, cache_len = dst_k, dst_v, new_len
    return stats


def test_step_chain_tiny_fp32_all_units():
    cfg = W.get_config("tiny")
    stats = _run_chain(cfg, range(cfg.n_layer), None, True)
    _note(f"tiny: {stats}")
    assert stats["exact"] + stats["band"] == cfg.n_layer * cfg.n_scale * cfg.n_seq * cfg.n_head


def test_step_chain_2b_512_sampled_units():
    cfg = W.get_config("2b_512")
    stats = _run_chain(cfg, [0, 17], [0, 5, 15], False)
    _note(f"2b_512: {stats}")
    assert stats["exact"] > 0


def test_step_chain_8b_shape_heavy_tailed_keys():
    """40-layer / 32-head shape with Student-t keys (near-ties, underflow) at its full size: all
    13 scales (up to 4096 queries) of two layers on all 512 units, three of them followed by the
    oracle through every scale."""
    cfg = W.get_config("8b_1024")
    stats = _run_chain(cfg, [0, 33], [0, 77, 511], False)
    _note(f"8b_1024: {stats}")
    assert stats["exact"] + stats["band"] == 2 * cfg.n_scale * 3


def test_step_chain_2b_1024_full_size_sampled_units():
    """The bench's own workload at its full size and in its launch configuration (16 x 16 units,
    all 13 scales up to 4096 queries) for one layer; two units followed by the oracle through
    every scale."""
    cfg = W.get_config("2b_1024")
    stats = _run_chain(cfg, [5], [3, 200], False)
    _note(f"2b_1024: {stats}")
    assert stats["exact"] + stats["band"] == cfg.n_scale * 2


def test_step_long_cache_and_other_shapes():
    """The routes of the ranking besides the one-launch kernel: a cache longer than the select holds in
    LDS (logits, finalise, select from global, compact); a cache of a length the one-launch kernel
    leaves to the logits + fused-select pair when there are few units (and the same with many
    queries, so that the pipelined attention follows the separate compaction); head_dim 64 in bf16;
    fp32 with head_dim 128."""
    for dtype, d, L, n_cur, budget in ((torch.bfloat16, 128, 13000, 40, 700), (torch.bfloat16, 128, 5000, 40, 500),
                                       (torch.bfloat16, 128, 4500, 200, 1000), (torch.bfloat16, 64, 900, 150, 333),
                                       (torch.float32, 128, 300, 50, 64)):
        _note(f"step dtype={dtype} d={d} L={L} n_cur={n_cur} budget={budget}")
        S, H = 1, 2
        shape = skv.Shape(S, H, d, dtype)
        q, kc, vc = (_rand(60 + i, (S, H, n_cur, d), dtype) for i in range(3))
        ks, vs = _rand(63, (S, H, L, d), dtype), _rand(64, (S, H, L, d), dtype)
        ws = torch.empty(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
        win = list(range(n_cur - 16, n_cur))
        kd = torch.zeros(S, H, budget + n_cur, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
        idx = torch.full((S, H, budget), -1, dtype=torch.int32, device=DEV)
        new_len = skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), win, ks.to(DEV), vs.to(DEV), L, budget,
                           kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        assert new_len == budget + n_cur
        g_idx = idx.cpu().numpy().reshape(S * H, budget)
        own = oracle.step(units(q), units(kc), units(vc), win, units(ks), units(vs), budget)
        for u in range(S * H):
            check_indices(g_idx[u], own["log_scores"][u], budget, own["idx"][u])
        ref = oracle.step(units(q), units(kc), units(vc), win, units(ks), units(vs), budget, force_idx=g_idx)
        assert np.array_equal(units(kd)[:, :new_len].double().numpy(), ref["k_dst"])
        check_output(out, ref["out"], dtype, f"step d={d} L={L}")


def test_step_is_reproducible_bit_for_bit_and_stays_inside_its_buffers():
    # no atomics on floats and a fixed reduction order everywhere: two runs give the same bits;
    # rows past the new cache length and the spare tail of the output keep their canary
    S, H, d, n_cur, L, budget = 2, 2, 128, 300, 500, 200
    dtype = torch.bfloat16
    _note("step reproducibility")
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (_rand(60 + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
    ks, vs = _rand(63, (S, H, L, d), dtype).to(DEV), _rand(64, (S, H, L, d), dtype).to(DEV)
    ws = torch.zeros(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    runs = []
    for _ in range(2):
        kd = torch.full((S, H, budget + n_cur + 9, d), 7.0, dtype=dtype, device=DEV); vd = torch.full_like(kd, 7.0)
        out = torch.full((S, H, n_cur, d), 7.0, dtype=dtype, device=DEV)
        idx = torch.full((S, H, budget), -1, dtype=torch.int32, device=DEV)
        new_len = skv.step(shape, q, kc, vc, list(range(n_cur - 16, n_cur)), ks, vs, L, budget, kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        assert new_len == budget + n_cur
        assert torch.all(kd[:, :, new_len:] == 7.0) and torch.all(vd[:, :, new_len:] == 7.0)
        runs.append((kd.clone(), vd.clone(), out.clone(), idx.clone()))
    for a, b in zip(*runs):
        assert torch.equal(a, b)
    kd, vd, out, idx = runs[0]
    assert torch.equal(kd[:, :, budget:budget + n_cur], kc) and torch.equal(vd[:, :, budget:budget + n_cur], vc)
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("n_cur", [48, 200])
def test_step_with_caches_that_are_views_of_larger_buffers(n_cur):
    # head stride > capacity * d, for the source and the destination alike
    S, H, d, L, budget = 2, 3, 128, 260, 100
    dtype = torch.bfloat16
    _note(f"step on strided cache views n_cur={n_cur}")
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (_rand(80 + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
    big_k, big_v = _rand(83, (S, H, L + 77, d), dtype).to(DEV), _rand(84, (S, H, L + 77, d), dtype).to(DEV)
    ks, vs = big_k[:, :, :L + 5], big_v[:, :, :L + 5]
    cap = budget + n_cur
    kd_big = torch.full((S, H, cap + 40, d), 3.0, dtype=dtype, device=DEV); vd_big = torch.full_like(kd_big, 3.0)
    kd, vd = kd_big[:, :, :cap], vd_big[:, :, :cap]
    out = torch.zeros(S, H, n_cur, d, dtype=dtype, device=DEV)
    idx = torch.zeros(S, H, budget, dtype=torch.int32, device=DEV)
    ws = torch.zeros(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    win = list(range(n_cur - 16, n_cur))
    new_len = skv.step(shape, q, kc, vc, win, ks, vs, L, budget, kd, vd, out, idx, ws)
    torch.cuda.synchronize()
    assert new_len == cap
    assert torch.all(kd_big[:, :, cap:] == 3.0) and torch.all(vd_big[:, :, cap:] == 3.0)
    g_idx = idx.cpu().numpy().reshape(S * H, budget)
    own = oracle.step(units(q), units(kc), units(vc), win, units(ks)[:, :L], units(vs)[:, :L], budget)
    for u in range(S * H):
        check_indices(g_idx[u], own["log_scores"][u], budget, own["idx"][u])
    ref = oracle.step(units(q), units(kc), units(vc), win, units(ks)[:, :L], units(vs)[:, :L], budget, force_idx=g_idx)
    assert np.array_equal(units(kd.contiguous()).double().numpy(), ref["k_dst"])
    assert np.array_equal(units(vd.contiguous()).double().numpy(), ref["v_dst"])
    check_output(out, ref["out"], dtype, "strided step")


def test_step_can_be_captured_in_a_graph_and_replayed():
    # The library neither allocates nor synchronises, so a step can be recorded into a HIP graph;
    # every replay (with eager work and synchronisations in between) must reproduce the eager bits.
    S, H, d, n_cur, L, budget = 1, 4, 128, 200, 300, 120
    dtype = torch.bfloat16
    _note("step under graph capture")
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (_rand(70 + i, (S, H, n_cur, d), dtype).to(DEV) for i in range(3))
    ks, vs = _rand(73, (S, H, L, d), dtype).to(DEV), _rand(74, (S, H, L, d), dtype).to(DEV)
    ws = torch.zeros(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    win = list(range(n_cur - 16, n_cur))
    mk = lambda: (torch.zeros(S, H, budget + n_cur, d, dtype=dtype, device=DEV),
                  torch.zeros(S, H, budget + n_cur, d, dtype=dtype, device=DEV),
                  torch.zeros(S, H, n_cur, d, dtype=dtype, device=DEV),
                  torch.zeros(S, H, budget, dtype=torch.int32, device=DEV))
    kd0, vd0, out0, idx0 = mk()
    skv.step(shape, q, kc, vc, win, ks, vs, L, budget, kd0, vd0, out0, idx0, ws)     # eager (also first-call set-up)
    torch.cuda.synchronize()
    kd, vd, out, idx = mk()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            skv.step(shape, q, kc, vc, win, ks, vs, L, budget, kd, vd, out, idx, ws)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in (kd, vd, out):
            t.fill_(5.0)                    # eager work between replays
        idx.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(kd, kd0) and torch.equal(vd, vd0), f"replay {rep}"
        assert torch.equal(out, out0) and torch.equal(idx, idx0), f"replay {rep}"


@pytest.mark.parametrize("n_cur", [40, 160])   # 160: the pipelined attention kernel with its two key segments
def test_step_edge_budgets(n_cur):
    dtype, S, H, d, L = torch.bfloat16, 1, 2, 128, 90
    _note(f"step edge budgets n_cur={n_cur}")
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (_rand(40 + i, (S, H, n_cur, d), dtype) for i in range(3))
    ks, vs = _rand(43, (S, H, L, d), dtype), _rand(44, (S, H, L, d), dtype)
    ws = torch.empty(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    win = list(range(n_cur - 16, n_cur))
    for budget in (0, 1, L - 1, L, L + 50):
        keep = min(budget, L)
        kd = torch.zeros(S, H, L + n_cur, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        # budget >= L and budget == 0 need no ranking, hence no workspace and no window
        use_ws = ws if 0 < budget < L else None
        new_len = skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), win if use_ws is not None else [],
                           ks.to(DEV), vs.to(DEV), L, budget, kd, vd, out, idx, use_ws)
        torch.cuda.synchronize()
        assert new_len == keep + n_cur
        ref = oracle.step(units(q), units(kc), units(vc), win, units(ks), units(vs), budget,
                          force_idx=idx.cpu().numpy().reshape(S * H, keep))
        if budget >= L:   # exact attention over the whole cache and the current map
            full = oracle.attend(units(q), torch.cat([units(ks), units(kc)], 1), torch.cat([units(vs), units(vc)], 1))
            assert np.abs(full - ref["out"]).max() < 1e-12
            assert np.array_equal(idx.cpu().numpy().reshape(S * H, keep), np.tile(np.arange(L), (S * H, 1)))
        check_output(out, ref["out"], dtype, f"budget {budget}")
        own = oracle.step(units(q), units(kc), units(vc), win, units(ks), units(vs), budget)
        for u in range(S * H):
            check_indices(idx.cpu().numpy().reshape(S * H, keep)[u], own["log_scores"][u], keep, own["idx"][u])


def test_step_sweep_of_sizes_around_the_tile_edges():
    """Seeded sweep of whole steps whose sizes sit on and next to the kernels' tile edges (32-row
    query blocks, 64-key tiles, 128-row query tiles, 256-key score chunks, the 128-row switch to
    the pipelined attention kernel), with windows scattered over the map, both dtypes and both
    head sizes; every unit is followed by the oracle."""
    rng = np.random.default_rng(20250519)
    edges_q = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 159, 160, 161, 255, 256, 257, 300]
    edges_l = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 700]
    for case in range(36):
        dtype = torch.bfloat16 if case % 3 else torch.float32
        d = 128 if case % 2 else 64
        S, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        n_cur, L = int(rng.choice(edges_q)), int(rng.choice(edges_l))
        budget = int(rng.choice([0, 1, max(1, L // 3), max(0, L - 1), L, L + 3]))
        keep = min(budget, L)
        n_win = int(rng.integers(1, min(16, n_cur) + 1))
        win = sorted(int(x) for x in rng.choice(n_cur, size=n_win, replace=False))
        _note(f"sweep case={case} dtype={dtype} d={d} S={S} H={H} n_cur={n_cur} L={L} budget={budget} n_win={n_win}")
        shape = skv.Shape(S, H, d, dtype)
        q, kc, vc = (_rand(900 + 7 * case + i, (S, H, n_cur, d), dtype) for i in range(3))
        ks, vs = (_rand(900 + 7 * case + 3 + i, (S, H, max(L, 1), d), dtype) for i in range(2))
        ws = torch.empty(skv.workspace_bytes(shape, max(L, 1), n_cur), dtype=torch.uint8, device=DEV)
        kd = torch.zeros(S, H, keep + n_cur, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        new_len = skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), win, ks.to(DEV), vs.to(DEV), L, budget,
                           kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        assert new_len == keep + n_cur
        g_idx = idx.cpu().numpy().reshape(S * H, keep)
        k_u, v_u = units(ks)[:, :L], units(vs)[:, :L]
        own = oracle.step(units(q), units(kc), units(vc), win, k_u, v_u, budget)
        for u in range(S * H):
            check_indices(g_idx[u], own["log_scores"][u], keep, own["idx"][u])
        ref = oracle.step(units(q), units(kc), units(vc), win, k_u, v_u, budget, force_idx=g_idx)
        assert np.array_equal(units(kd)[:, :new_len].double().numpy(), ref["k_dst"])
        assert np.array_equal(units(vd)[:, :new_len].double().numpy(), ref["v_dst"])
        check_output(out, ref["out"], dtype, f"sweep case {case}")


def test_step_random_shapes_follow_the_oracle():
    """Seeded whole steps at sizes drawn at random rather than at tile edges (maps of 1-700 tokens,
    caches of 0-2500 rows, budgets from 0 to beyond the cache, windows in any order, three logit
    scales, both dtypes and head sizes), with canary rows behind the new cache; every unit is
    followed by the oracle."""
    rng = np.random.default_rng(20251128)
    for case in range(60):
        dtype = torch.bfloat16 if rng.random() < 0.8 else torch.float32
        d = 128 if rng.random() < 0.7 else 64
        S, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        n_cur = int(rng.choice([rng.integers(1, 40), rng.integers(1, 200), rng.integers(100, 700)]))
        L = int(rng.choice([rng.integers(0, 40), rng.integers(0, 600), rng.integers(300, 2500)]))
        budget = int(rng.choice([0, 1, rng.integers(0, L + 2), rng.integers(0, L + 2), max(0, L - 1), L, L + 3]))
        keep = min(budget, L)
        n_win = int(rng.integers(1, min(16, n_cur) + 1))
        win = [int(x) for x in rng.choice(n_cur, size=n_win, replace=False)]
        logit_scale = float(rng.choice([0.3, 1.0, 2.5]))
        pad = int(rng.integers(0, 4))
        _note(f"random step case={case} dtype={dtype} d={d} S={S} H={H} n_cur={n_cur} L={L} budget={budget} "
              f"n_win={n_win} scale={logit_scale} pad={pad}")
        shape = skv.Shape(S, H, d, dtype)
        q, kc, vc = (_rand(5000 + 7 * case + i, (S, H, n_cur, d), dtype, logit_scale if i < 2 else 1.0) for i in range(3))
        ks = _rand(5000 + 7 * case + 3, (S, H, max(L, 1), d), dtype, logit_scale)
        vs = _rand(5000 + 7 * case + 4, (S, H, max(L, 1), d), dtype)
        ws = torch.empty(skv.workspace_bytes(shape, max(L, 1), n_cur), dtype=torch.uint8, device=DEV)
        kd = torch.full((S, H, keep + n_cur + pad, d), 3.0, dtype=dtype, device=DEV); vd = torch.full_like(kd, 3.0)
        out = torch.full((S, H, n_cur, d), float("nan"), dtype=dtype, device=DEV)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        new_len = skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), win, ks.to(DEV), vs.to(DEV), L, budget,
                           kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        assert new_len == keep + n_cur
        assert torch.all(kd[:, :, new_len:] == 3.0) and torch.all(vd[:, :, new_len:] == 3.0)
        g_idx = idx.cpu().numpy().reshape(S * H, keep)
        k_u, v_u = units(ks)[:, :L], units(vs)[:, :L]
        own = oracle.step(units(q), units(kc), units(vc), win, k_u, v_u, budget)
        for u in range(S * H):
            check_indices(g_idx[u], own["log_scores"][u], keep, own["idx"][u])
        ref = oracle.step(units(q), units(kc), units(vc), win, k_u, v_u, budget, force_idx=g_idx)
        assert np.array_equal(units(kd)[:, :new_len].double().numpy(), ref["k_dst"])
        assert np.array_equal(units(vd)[:, :new_len].double().numpy(), ref["v_dst"])
        check_output(out, ref["out"], dtype, f"random step case {case}")


def test_attend_heavy_tailed_keys_at_random_shapes():
    """The pipelined attention kernel on Student-t keys scaled by 1 to 10: rows whose later scores
    sit a little, far, or too far above the first tile's maximum, so that workgroups with and
    without the repeat pass (and both kinds in one launch) are compared with the oracle."""
    rng = np.random.default_rng(20251129)
    dtype, d = torch.bfloat16, 128
    for case in range(24):
        S, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        n_q, kv = int(rng.integers(129, 700)), int(rng.integers(65, 3000))
        scale = float(rng.choice([1.0, 3.0, 6.0, 10.0]))
        _note(f"heavy-tailed attend case={case} S={S} H={H} n_q={n_q} kv={kv} scale={scale}")
        q = _rand(7000 + 3 * case, (S, H, n_q, d), dtype)
        k = (W.student_t_tensor(W.stream_key(7001, case), W.stream_key(7002, case), (S, H, kv, d)) * scale).to(dtype)
        v = _rand(7000 + 3 * case + 2, (S, H, kv, d), dtype)
        out = torch.full((S, H, n_q, d), float("nan"), dtype=dtype, device=DEV)
        skv.attend(skv.Shape(S, H, d, dtype), q.to(DEV), k.to(DEV), v.to(DEV), kv, out)
        torch.cuda.synchronize()
        check_output(out, oracle.attend(units(q), units(k), units(v)), dtype, f"heavy-tailed attend case {case}")


def test_step_one_hot_pattern_selects_its_argmax():
    dtype, S, H, d, L, n_cur = torch.bfloat16, 1, 2, 128, 400, 32
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (_rand(50 + i, (S, H, n_cur, d), dtype, 0.1) for i in range(3))
    ks, vs = _rand(53, (S, H, L, d), dtype, 0.1), _rand(54, (S, H, L, d), dtype)
    direction = torch.nn.functional.normalize(W.normal_tensor(W.stream_key(55, 0), (d,)), dim=0)
    win = [3, 10, 31]
    q[:, :, win] = (5.0 * direction).to(dtype)
    ks[:, 0, 123] = (40.0 * direction).to(dtype); ks[:, 1, 377] = (40.0 * direction).to(dtype)
    ws = torch.empty(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    for budget in (1, 7):
        kd = torch.zeros(S, H, budget + n_cur, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
        idx = torch.zeros(S, H, budget, dtype=torch.int32, device=DEV)
        skv.step(shape, q.to(DEV), kc.to(DEV), vc.to(DEV), win, ks.to(DEV), vs.to(DEV), L, budget, kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        got = idx.cpu().numpy()
        assert 123 in got[0, 0] and 377 in got[0, 1]


# ------------------------------------------- full-size, bench launch shapes --

def test_final_scale_full_size_sampled_against_oracle():
    """The 64x64 scale at the bench's shape (16 sequences x 16 heads, 4096
    queries, 6489 cached rows), all four budgets; the oracle checks sampled
    units and, within them, sampled query rows."""
    cfg = W.get_config("final_scale")
    dtype = torch.bfloat16
    S, H, d = cfg.n_seq, cfg.n_head, cfg.head_dim
    shape = skv.Shape(S, H, d, dtype)
    case = W.make_final_scale_case(cfg, DEV)
    n_cur, L = case.q.shape[2], case.k_hist.shape[2]
    assert (n_cur, L) == (4096, 6489)
    win = W.window_indices(cfg, n_cur)
    ws = torch.empty(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
    sample_units = [0, 101, 255]
    sample_rows = [0, 1, 777, 2048, 4095]
    out = torch.empty(S, H, n_cur, d, dtype=dtype, device=DEV)
    for budget in W.final_scale_budgets(cfg):
        _note(f"final scale budget={budget}")
        keep = min(budget, L)
        kd = torch.zeros(S, H, keep + n_cur, d, dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        new_len = skv.step(shape, case.q, case.k_cur, case.v_cur, win, case.k_hist, case.v_hist, L, budget,
                           kd, vd, out, idx, ws)
        torch.cuda.synchronize()
        assert new_len == keep + n_cur
        g_idx = idx.cpu().numpy().reshape(S * H, keep)
        assert np.all(np.diff(g_idx, axis=1) > 0) and g_idx.min() >= 0 and g_idx.max() < L   # all units: valid lists
        boosted = case.boosted.cpu().numpy().reshape(S * H, L)
        for u in sample_units:
            qu, khu = units(case.q)[u:u + 1], units(case.k_hist)[u:u + 1]
            _, ls_ref = oracle.score(qu[:, win], khu)
            o_idx = oracle.select(ls_ref, budget)
            check_indices(g_idx[u], ls_ref[0], keep, o_idx[0])
            if budget < L and keep >= boosted[u].sum():
                # the dominant keys are (nearly all) kept: a property of this workload, not of parity
                assert np.isin(np.nonzero(boosted[u])[0], g_idx[u]).mean() > 0.9
            k_new = oracle.compact(khu, g_idx[u:u + 1], units(case.k_cur)[u:u + 1])
            v_new = oracle.compact(units(case.v_hist)[u:u + 1], g_idx[u:u + 1], units(case.v_cur)[u:u + 1])
            assert np.array_equal(units(kd)[u, :new_len].double().numpy(), k_new[0])
            assert np.array_equal(units(vd)[u, :new_len].double().numpy(), v_new[0])
            ref = oracle.attend(qu[:, sample_rows], k_new, v_new)
            check_output(units(out)[u:u + 1, sample_rows], ref, dtype, f"final scale u{u} b{budget}")
