#!/usr/bin/env python3
"""ScaleKV hot-path benchmark on one MI355X.

One "step" = the whole multi-scale sequence of one image batch: for each of the
13 scales and each of the 32 layers, one scalekv_step call (score -> select ->
compact -> attend) over seeded synthetic Q/K/V of the Infinity-2B shape at
1024^2, batch 8 with classifier-free-guidance rows (16 sequences).  All inputs
and caches are resident in HBM before the timed region starts.

Prints ONE JSON line: the headline metric (ms per 13-scale image batch), the
roofline of the dominant kernel (the bf16 MFMA attention) from HIP events
recorded around its launches, on the launch stream, inside the timed region;
per-stage times and bandwidths from one more, untimed pass with an event at every
stage boundary; and the fp64 CPU oracle timed on a bounded sample of the same
workload.

--variant picks what each (layer, scale) call is; the default is the graded path:
  scalekv   scalekv_step: score -> select -> compact -> attend, drafter/refiner budgets
  literal   scalekv_step_append_first: Sec. 3.3 in its literal order (append, attend, then
            score over history and map, pooled scores, window kept), 4x4 patch-centroid window
  pyramid   scalekv_step with the per-layer pyramid budgets of scalekv_pyramid_budgets
  sliding   scalekv_select_positional (most recent tokens) -> compact -> attend, uniform budget
  sinks     the same with the first 16 positions kept as well
The last three are the comparison policies of Sec. 4.1 at the same total budget: their cost,
not their quality.

--cases L,B,N[;L,B,N...] runs nothing but a few scalekv_step calls of the listed shapes
(cache_len, budget, n_cur) on random inputs after a 1 GiB device-to-device copy, for use under
rocprofv3: the copy calibrates the hardware byte counters (FETCH_SIZE, WRITE_SIZE), and the n-th
group of the library's kernels in the trace belongs to the n-th case.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch of the pipelined attention kernel (which also appends the map's K/V) at
# 16 x 16 units, d128, bf16, keyed by (n_cur, keep): rocprofv3 --pmc FETCH_SIZE (KiB, scaled by
# 2.0: what the same counter reads for a plain copy of known size) plus --pmc WRITE_SIZE (KiB,
# scale 1.0), three launches each, inside scalekv_step.  The commands and the full per-kernel table are in profiles/step_hbm_traffic.md.
ATTEND_PIPE_TRAFFIC = {
    (144, 46): 63.0e6, (144, 9): 58.2e6,
    (256, 82): 125.9e6, (256, 16): 119.6e6,
    (400, 146): 191.2e6, (400, 29): 177.0e6,
    (576, 246): 283.4e6, (576, 49): 262.3e6,
    (1024, 390): 488.1e6, (1024, 78): 459.5e6,
    (1600, 646): 841.4e6, (1600, 129): 759.3e6,
    (2304, 1046): 1304.6e6, (2304, 209): 1152.4e6,
    (4096, 1622): 1943.3e6, (4096, 324): 1855.5e6,
}


VARIANTS = ("scalekv", "literal", "pyramid", "sliding", "sinks", "calibrated")
# stages between consecutive events of one call, per variant
# ("score" holds the whole ranking where the selection kernel streams the keys itself: one launch;
# "select" is then only what lies between two events)
STAGES = {
    "scalekv": ("score", "select", "compact", "attend"),
    "pyramid": ("score", "select", "compact", "attend"),
    "calibrated": ("score", "select", "compact", "attend"),
    "literal": ("append", "attend", "score+select", "compact"),
    "sliding": ("select", "compact", "attend"),
    "sinks": ("select", "compact", "attend"),
}
N_SINK = 16


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


class HipEvents:
    """Raw hipEvent_t handles from the same HIP runtime the library uses."""

    def __init__(self, lib):
        self.lib = lib
        lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pool = []

    def block(self, n: int, only=None):
        """n slots; with `only`, just those slots hold an event and the rest stay NULL"""
        arr = (ctypes.c_void_p * n)()
        for i in (range(n) if only is None else only):
            e = ctypes.c_void_p()
            rc = self.lib.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            arr[i] = e
        self.pool.append(arr)
        return arr

    def elapsed_ms(self, a, b) -> float:
        out = ctypes.c_float(0)
        rc = self.lib.hipEventElapsedTime(ctypes.byref(out), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(out.value)

    def destroy(self):
        for arr in self.pool:
            for e in arr:
                if e:
                    self.lib.hipEventDestroy(e)
        self.pool = []


def cpu_baseline(cfg, W, seconds_hint: float = 20.0):
    """The oracle, as it stands, on a bounded sample: every scale of two layers -- one that is a
    drafter and one that is a refiner at the last scale, where almost all of the work is -- for two
    (sequence, head) units per host thread each.  Extrapolated by unit count, the two layers
    weighted by the number of drafter and refiner layers."""
    import oracle
    n_thr = oracle.num_threads()
    K = cfg.n_scale
    units = list(range(min(2 * n_thr, cfg.n_seq * cfg.n_head)))
    table = W.budget_table(cfg)
    roles = W.layer_roles(cfg, K)
    n_d = sum(roles)
    layers = [0]
    if 0 < n_d < cfg.n_layer:
        layers = [roles.index(True), roles.index(False)]
    # inputs are generated before the clock starts
    chains = []
    for layer in layers:
        kp, vp = W.make_prefix(cfg, layer, "cpu", units)
        steps = []
        for k in range(1, K + 1):
            x = W.make_step_inputs(cfg, layer, k, "cpu", units)
            steps.append((x.q.double().numpy(), x.k_cur.double().numpy(), x.v_cur.double().numpy(),
                          W.window_indices(cfg, cfg.n_tokens(k)), table[layer][k - 1]))
        chains.append((kp.double().numpy(), vp.double().numpy(), steps))
    secs = []
    for src_k, src_v, steps in chains:
        t0 = time.perf_counter()
        for (q, kc, vc, win, budget) in steps:
            r = oracle.step(q, kc, vc, win, src_k, src_v, budget)
            src_k, src_v = r["k_dst"], r["v_dst"]
        secs.append(time.perf_counter() - t0)
    U = cfg.n_seq * cfg.n_head
    weights = [n_d, cfg.n_layer - n_d] if len(layers) == 2 else [cfg.n_layer]
    est_ms = sum(t * w for t, w in zip(secs, weights)) * 1e3 * U / len(units)
    which = (f"layers {layers[0]} (drafter at the last scale, weight {weights[0]}) and {layers[1]} "
             f"(refiner there, weight {weights[1]})") if len(layers) == 2 else f"layer {layers[0]}"
    return {
        "value": est_ms, "unit": f"ms per {K}-scale image batch (extrapolated by unit count)",
        "cores": n_thr, "kind": "oracle",
        "sample": f"all {K} scales of {which} for {len(units)} of {U} (sequence, head) units, two per thread; "
                  f"{sum(secs):.2f} s measured, scaled by {U}/{len(units)} units and the layer weights",
        "sample_seconds": sum(secs),
    }


def final_scale_sweep(args, torch, skv, W, cfg) -> int:
    """--config final_scale: only the 64x64 scale of the 2b_1024 shape, one scalekv_step per
    budget (5 / 10 / 20 / 100 % of the 6489 cached rows); the 100 % case is uncompressed
    attention over 10585 keys.  Median of 10 repetitions per budget, HIP events on the launch
    stream.  One JSON line; `value` is the 10 % case."""
    dev, dtype = "cuda", torch.bfloat16
    S, H, d = cfg.n_seq, cfg.n_head, cfg.head_dim
    U = S * H
    shape = skv.Shape(S, H, d, dtype)
    case = W.make_final_scale_case(cfg, dev)
    n_cur, L = case.q.shape[2], case.k_hist.shape[2]
    win = W.window_indices(cfg, n_cur)
    ws = torch.empty(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=dev)
    out = torch.empty(S, H, n_cur, d, dtype=dtype, device=dev)
    events = HipEvents(skv.lib())
    hip = skv.lib()
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    stream_ptr = torch.cuda.current_stream().cuda_stream
    rows = []
    for frac, budget in zip(W.FINAL_SCALE_BUDGET_FRACS, W.final_scale_budgets(cfg)):
        keep = min(budget, L)
        kd = torch.empty(S, H, keep + n_cur, d, dtype=dtype, device=dev); vd = torch.empty_like(kd)
        call = skv.PreparedStep(shape, case.q, case.k_cur, case.v_cur, win, case.k_hist, case.v_hist, L, budget,
                                kd, vd, out, None, ws)
        for _ in range(max(1, args.warmup)):
            call(stream_ptr)
        reps = 10
        ev = events.block(reps + 1)
        hip.hipEventRecord(ev[0], stream_ptr)
        for r in range(reps):
            call(stream_ptr)
            hip.hipEventRecord(ev[r + 1], stream_ptr)
        torch.cuda.synchronize()
        ms = sorted(events.elapsed_ms(ev[r], ev[r + 1]) for r in range(reps))
        med = 0.5 * (ms[reps // 2 - 1] + ms[reps // 2])
        flops = 4.0 * n_cur * (keep + n_cur) * d * U
        rows.append({"budget_frac": frac, "keep": keep, "kv_len": keep + n_cur, "ms_median": med, "ms_min": ms[0],
                     "attend_tflop": flops / 1e12, "step_tflops": flops / (med * 1e-3) / 1e12})
        log(f"budget {frac:.0%}: keep {keep}, {med:.3f} ms per step ({rows[-1]['step_tflops']:.0f} TFLOP/s on the attention flops)")
        del kd, vd
    events.destroy()
    ten = next(r for r in rows if abs(r["budget_frac"] - 0.10) < 1e-9)
    full = rows[-1]
    print(json.dumps({
        "metric": "ScaleKV step ms at the final 64x64 scale, 10 % budget", "value": ten["ms_median"], "unit": "ms",
        "n_gpus": 1, "steps": 10, "warmup": max(1, args.warmup), "ms_per_step": ten["ms_median"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"final_scale: {S} sequences x {H} heads x d{d}, {n_cur} queries against {L} cached rows "
                               f"(1 % dominant keys), budgets 5/10/20/100 %, window {cfg.window}"},
        "sweep": rows,
        "speedup_10pct_over_uncompressed": full["ms_median"] / ten["ms_median"],
    }), flush=True)
    return 0


def run_cases(args, torch, skv) -> int:
    """--cases: a calibration copy, then `--reps` scalekv_step calls per listed shape."""
    dev, dt = "cuda", torch.bfloat16
    S, H, d = args.case_seqs, args.case_heads, 128
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(args.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    shape = skv.Shape(S, H, d, dt)
    g = torch.Generator(device=dev).manual_seed(0)
    rnd = lambda rows: torch.randn(S, H, rows, d, device=dev, dtype=torch.float32, generator=g).to(dt)
    for case in args.cases.split(";"):
        L, budget, n = (int(x) for x in case.split(","))
        q, kc, vc, ks, vs = rnd(n), rnd(n), rnd(n), rnd(L), rnd(L)
        keep = min(budget, L)
        kd = torch.empty(S, H, keep + n, d, device=dev, dtype=dt)
        vd = torch.empty_like(kd)
        out = torch.empty_like(q)
        ws = torch.empty(skv.workspace_bytes(shape, L, n), dtype=torch.uint8, device=dev)
        win = list(range(max(0, n - 16), n))
        for _ in range(args.reps):
            skv.step(shape, q, kc, vc, win, ks, vs, L, budget, kd, vd, out, None, ws)
        torch.cuda.synchronize()
        print(f"ran {args.reps} steps: cache_len={L} keep={keep} n_cur={n} units={S * H}", flush=True)
        del q, kc, vc, ks, vs, kd, vd, out, ws
    return 0


def attend_alone(args, torch, skv) -> int:
    """--attend-alone N_Q,KV_LEN: the pipelined attention kernel by itself (scalekv_attend, one key
    segment, nothing else to carry) on 16 x 16 units of seeded normal data, or of zeros with
    --zero-keys (the same instruction stream switching fewer bits).  With --library it runs one of
    the measurement-only builds of `python -m paper_2505_19602_amd.build --variant ...`, whose
    results are wrong on purpose: timing only.  One JSON line."""
    import workloads as W
    dev, dt = "cuda", torch.bfloat16
    S, H, d = args.case_seqs, args.case_heads, 128
    n_q, kv = (int(x) for x in args.attend_alone.split(","))
    shape = skv.Shape(S, H, d, dt)
    mk = lambda key, rows: W.normal_tensor(W.stream_key(4242, key), (S, H, rows, d), dev).to(dt)
    q, k, v = mk(1, n_q), mk(2, kv), mk(3, kv)
    if args.zero_keys:
        k.zero_()
    out = torch.empty_like(q)
    for _ in range(3):
        skv.attend(shape, q, k, v, kv, out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(args.reps):
        skv.attend(shape, q, k, v, kv, out)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.reps
    flops = 4.0 * n_q * kv * d * S * H
    line = {"mode": "attend-alone", "library": os.path.basename(skv.lib_path()), "zero_keys": bool(args.zero_keys),
            "units": S * H, "n_q": n_q, "kv_len": kv, "reps": args.reps, "ms": ms,
            "tflops": flops / (ms * 1e-3) / 1e12, "frac_of_bf16_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    if args.timeline:
        line["timeline"] = timeline_summary(skv, (n_q + 127) // 128 * S * H)
    print(json.dumps(line), flush=True)
    return 0


def attend_clock_leg():
    """The clock the chip holds under the attention kernel, per XCD: a child process runs
    `--attend-alone 4096,5718 --timeline` with the measurement build of the library whose
    workgroups read the shader clock counter (python -m paper_2505_19602_amd.build --variant
    timeline); None if that build is not there.  Outside the timed region."""
    import subprocess
    lib = os.path.join(ROOT, "paper_2505_19602_amd", "libscalekv_timeline.so")
    if not os.path.exists(lib):
        return None
    cmd = [sys.executable, os.path.abspath(__file__), "--attend-alone", "4096,5718", "--reps", "5", "--timeline",
           "--library", lib]
    try:
        res = subprocess.run(cmd, capture_output=True, text=True, timeout=180, cwd=ROOT)
        line = json.loads(res.stdout.strip().splitlines()[-1])
        mhz = [x["clock_counter_mhz"] for x in line["timeline"]["per_xcd"]]
        mean = sum(mhz) / len(mhz)
        peak = PEAK_BF16_TFLOPS * mean / 2400.0
        return {"shape": "attention kernel alone, 4096 queries x 5718 keys x 256 units", "tflops": line["tflops"],
                "mhz_per_xcd": mhz, "mhz_mean": mean, "matrix_peak_at_that_clock_tflops": peak,
                "frac_of_that_peak": line["tflops"] / peak, "idle_at_the_end": line["timeline"]["idle_at_the_end"],
                "note": "shader clock counter over 100 MHz counter, summed over each XCD's workgroups; the vendor peak "
                        "assumes 2400 MHz; idle_at_the_end = share of the launch the XCDs, on average, wait for the slowest"}
    except Exception as exc:
        return {"error": f"{type(exc).__name__}: {exc}"[:300]}


def timeline_summary(skv, n_wg: int) -> dict:
    """Per-workgroup records of the last attention launch, from a library built with
    `--variant timeline` (four readings of the 100 MHz counter, the hardware id register and two readings of
    the shader clock counter per workgroup), summed up per XCD: hardware hands workgroup i to XCD i mod 8."""
    import ctypes

    import numpy as np
    L = skv.lib()
    if not hasattr(L, "scalekv_timeline_read"):
        raise SystemExit("--timeline needs --library <a build made with --variant timeline>")
    rec = np.zeros((n_wg, 7), dtype=np.uint64)
    rc = L.scalekv_timeline_read(rec.ctypes.data_as(ctypes.c_void_p), ctypes.c_int(n_wg))
    if rc != 0:
        raise SystemExit(f"scalekv_timeline_read returned {rc} (the build keeps records of at most 8192 workgroups; "
                         f"this launch has {n_wg})")
    t = (rec[:, :4].astype(np.int64) - int(rec[:, 0].min())) * 0.01  # us since the first workgroup started
    hw = rec[:, 4].astype(np.int64)
    xcd = np.arange(n_wg) % 8
    cu = (((hw >> 13) & 7) * 2 + ((hw >> 12) & 1)) * 16 + ((hw >> 8) & 15)  # within the XCD
    span = float(t[:, 3].max())
    dur = t[:, 3] - t[:, 0]
    n_cu = sum(len(np.unique(cu[xcd == x])) for x in range(8))
    cyc = (rec[:, 6] - rec[:, 5]).astype(np.float64)  # shader clock counter over the workgroup's life
    per_xcd = [{"xcd": x, "workgroups": int((xcd == x).sum()), "mean_wg_us": round(float(dur[xcd == x].mean()), 1),
                "last_end_us": round(float(t[xcd == x, 3].max()), 1),
                "clock_counter_mhz": round(float(cyc[xcd == x].sum() / dur[xcd == x].sum()), 1)}
               for x in range(8) if (xcd == x).any()]
    ends = [p["last_end_us"] for p in per_xcd]
    return {"workgroups": n_wg, "compute_units": n_cu, "span_us": round(span, 1),
            "wg_us": {"mean": round(float(dur.mean()), 1), "min": round(float(dur.min()), 1), "max": round(float(dur.max()), 1)},
            "start_to_first_tile_us": round(float((t[:, 1] - t[:, 0]).mean()), 2),
            "tile_loop_us": round(float((t[:, 2] - t[:, 1]).mean()), 1),
            "loop_end_to_end_us": round(float((t[:, 3] - t[:, 2]).mean()), 2),
            "slot_occupancy": round(float(dur.sum() / (2 * n_cu * span)), 3),
            "tile_loop_share_of_slot_time": round(float((t[:, 2] - t[:, 1]).sum() / (2 * n_cu * span)), 3),
            "per_xcd": per_xcd,
            "idle_at_the_end": round(float(1.0 - np.mean(ends) / span), 4)}


def parity_replay(torch, skv, W, cfg, shape, inputs, prefix, bufs, table, lens_before_last, windows, ws,
                  n_units: int = 2, n_rows: int = 48):
    """After the timed region: the last scale's call of one drafter layer and one refiner layer is
    issued once more with the very arguments the timed passes used (same shapes, same launch
    configuration, same source cache, which the passes leave intact), now also returning its
    indices, and sampled units are replayed through the fp64 oracle: indices by the margin rule,
    the new cache bit for bit, the attention output on sampled query rows."""
    import numpy as np
    import oracle
    K, S, H, d = cfg.n_scale, cfg.n_seq, cfg.n_head, cfg.head_dim
    U = S * H
    n_cur = cfg.n_tokens(K)
    roles = W.layer_roles(cfg, K)
    layers = sorted({roles.index(True), roles.index(False)}) if (True in roles and False in roles) else [0]
    units = [int(u) for u in np.linspace(0, U - 1, n_units).round()]
    rows = sorted({int(r) for r in np.linspace(0, n_cur - 1, n_rows).round()})
    stats = dict(layers=layers, units=units, query_rows=len(rows), exact=0, band=0, kv_bit_exact=True, max_err=0.0,
                 mean_err=0.0, tolerance="indices: equal where the keep-th / (keep+1)-th score margin exceeds 1e-4, "
                 "else inside the band; K'/V' bit-exact; output 2e-2 max-abs, 1e-2 mean-abs (bf16)")
    flat = lambda t: t.reshape(U, t.shape[2], d)
    errs = []
    for l in layers:
        x = inputs[(l, K)]
        src = bufs[l][(K - 1) % 2] if K > 1 else prefix[l]
        dst = bufs[l][K % 2]
        L, budget = lens_before_last[l], table[l][K - 1]
        keep = min(budget, L)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=x.q.device)
        out = torch.empty_like(x.q)
        new_len = skv.step(shape, x.q, x.k_cur, x.v_cur, windows[K], src[0], src[1], L, budget, dst[0], dst[1], out, idx, ws)
        torch.cuda.synchronize()
        g_idx = idx.cpu().numpy().reshape(U, keep)[units]
        q_u, kc_u, vc_u = (flat(t)[units].cpu() for t in (x.q, x.k_cur, x.v_cur))
        ks_u, vs_u = (flat(t[:, :, :L])[units].cpu() for t in src)
        if 0 < keep < L:
            _, ls = oracle.score(q_u[:, windows[K]], ks_u)
            own = oracle.select(ls, budget)
            for i in range(len(units)):
                order = np.sort(ls[i])[::-1]
                la, lb = order[keep - 1], order[keep]
                if lb - la < np.log1p(-1e-4):
                    assert np.array_equal(g_idx[i], own[i]), f"parity: indices differ at a wide margin (layer {l}, unit {units[i]})"
                    stats["exact"] += 1
                else:
                    chosen = np.zeros(L, dtype=bool); chosen[g_idx[i]] = True
                    assert np.all(chosen[ls[i] > la + np.log1p(1e-4)]) and np.all(ls[i][chosen] >= la + np.log1p(-1e-4)), \
                        f"parity: invalid choice inside the near-tie band (layer {l}, unit {units[i]})"
                    stats["band"] += 1
        k_new = oracle.compact(ks_u, g_idx, kc_u)
        v_new = oracle.compact(vs_u, g_idx, vc_u)
        got_k, got_v = (flat(t[:, :, :new_len])[units].cpu().double().numpy() for t in dst)
        stats["kv_bit_exact"] = bool(stats["kv_bit_exact"] and np.array_equal(got_k, k_new) and np.array_equal(got_v, v_new))
        ref = oracle.attend(q_u[:, rows], k_new, v_new)
        got = flat(out)[units][:, rows].float().cpu().numpy().astype(np.float64)
        errs.append(np.abs(got - ref))
    err = np.concatenate([e.ravel() for e in errs])
    stats["max_err"], stats["mean_err"] = float(err.max()), float(err.mean())
    stats["ok"] = bool(stats["kv_bit_exact"] and stats["max_err"] <= 2e-2 and stats["mean_err"] <= 1e-2)
    return stats


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="2b_1024")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stage-pass", action="store_true",
                    help="skip the extra, untimed pass that records events at every stage boundary")
    ap.add_argument("--no-graph-pass", action="store_true",
                    help="skip the extra leg that replays the whole sequence from one captured HIP graph")
    ap.add_argument("--variant", default="scalekv", choices=VARIANTS)
    ap.add_argument("--pool-w", type=int, default=7, help="score pooling width of --variant literal")
    ap.add_argument("--shared-inputs", action="store_true",
                    help="reuse layer 0's Q/K/V in every layer (less memory, faster set-up)")
    ap.add_argument("--no-clock-leg", action="store_true",
                    help="skip the child run that reads the clock the attention kernel runs at (needs the timeline build)")
    ap.add_argument("--no-parity", action="store_true",
                    help="skip the replay of sampled last-scale units through the CPU oracle after the timed region")
    ap.add_argument("--cases", default=None,
                    help="cache_len,budget,n_cur[;...]: only run these step shapes on random inputs (for rocprofv3)")
    ap.add_argument("--reps", type=int, default=3, help="calls per shape of --cases / timed calls of --attend-alone")
    ap.add_argument("--attend-alone", default=None, help="N_Q,KV_LEN: time the pipelined attention kernel by itself")
    ap.add_argument("--zero-keys", action="store_true", help="--attend-alone with all keys zero")
    ap.add_argument("--timeline", action="store_true",
                    help="--attend-alone with a --variant timeline build: per-XCD summary of the workgroups' start and end times")
    ap.add_argument("--library", default=None,
                    help="path of a measurement-only build of the library to load instead of the in-tree one")
    ap.add_argument("--case-seqs", type=int, default=16)
    ap.add_argument("--case-heads", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    if args.library:
        if not (args.attend_alone or args.cases):
            print("--library is for --attend-alone / --cases runs only: those builds give wrong results", file=sys.stderr)
            return 2
        os.environ["SCALEKV_LIBRARY"] = os.path.abspath(args.library)
    import torch
    import paper_2505_19602_amd as skv
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda"
    if args.attend_alone:
        return attend_alone(args, torch, skv)
    if args.cases:
        return run_cases(args, torch, skv)
    cfg = W.get_config(args.config)
    if cfg.name == "final_scale":
        return final_scale_sweep(args, torch, skv, W, cfg)
    dtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    S, H, d, Lyr, K = cfg.n_seq, cfg.n_head, cfg.head_dim, cfg.n_layer, cfg.n_scale
    U = S * H
    e = cfg.elem_bytes
    shape = skv.Shape(S, H, d, dtype)
    cap = W.dst_capacity(cfg)
    table = W.budget_table(cfg)
    # total retained fraction of the drafter/refiner table: the uniform budget of the comparison policies
    uniform_frac = (cfg.n_drafter * cfg.drafter_frac + (Lyr - cfg.n_drafter) * cfg.refiner_frac) / Lyr
    if args.variant == "literal":   # the cache buffer also holds the map before pruning
        cap = max(cap, max(W.c_full(cfg, k) + cfg.n_tokens(k) for k in range(1, cfg.first_compressed_scale)),
                  max(16 + max(r[k - 2] for r in table) + cfg.n_tokens(k) for k in range(2, K + 1)))
    if args.variant == "pyramid":
        cap = max(int(2 * uniform_frac * W.c_full(cfg, k) + 1) + cfg.n_tokens(k) for k in range(1, K + 1))
        cap = max(cap, W.dst_capacity(cfg))
    log(f"{skv.version()}  workload {cfg.name}: S={S} H={H} d={d} layers={Lyr} scales={K} cap={cap}")

    # ---- resident state: prefix caches, ping-pong caches, per-(layer, scale) inputs
    t_setup = time.perf_counter()
    prefix = [W.make_prefix(cfg, l, dev) for l in range(Lyr)]
    inputs = {}
    for k in range(1, K + 1):
        for l in range(Lyr):
            if args.shared_inputs and l > 0:
                inputs[(l, k)] = inputs[(0, k)]
            else:
                inputs[(l, k)] = W.make_step_inputs(cfg, l, k, dev)
        torch.cuda.synchronize()
        log(f"inputs for scale {k}/{K} ready ({torch.cuda.memory_allocated() / 2**30:.1f} GiB resident)")
    calibration = None
    if args.variant == "calibrated":
        # Sec. 3.2 on this workload's own tensors: ASI of every (layer, scale) pair on the uncompressed
        # cache (Eq. 2), the lowest-Z pairs become drafters (Eq. 3), Eq. 4 splits the uniform budget.
        # Same number of drafter pairs and same mean budget as the seeded drafter/refiner table; the
        # paper's B_r(0) and delta (600 and 70 at a uniform budget of 650) scaled to this uniform budget.
        n_samp, top_k = 16, 64
        b_uni = max(1, int(uniform_frac * W.c_full(cfg, K) + 0.5))
        b_r0, delta = b_uni * 600 // 650, max(1, (b_uni * 70 * 13) // (650 * K))
        full_len = W.c_full(cfg, K) + cfg.n_tokens(K)
        ws_asi = torch.empty(skv.workspace_bytes(shape, full_len, n_samp), dtype=torch.uint8, device=dev)
        asi_dev = torch.zeros(Lyr, K, 3, dtype=torch.float32, device=dev)
        t_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        asi_ms = 0.0
        for l in range(Lyr):
            hist = [prefix[l][0]]
            for k in range(1, K + 1):
                x = inputs[(l, k)]
                case = W.assemble_asi_case(hist, x.q, x.k_cur, n_samp)
                terms = torch.empty(S, H, case.q_samp.shape[2], 2, dtype=torch.float32, device=dev)
                t_ev[0].record()
                skv.asi(shape, case.q_samp, case.k_all, case.hist_len, case.cur_len, top_k, terms, asi_dev[l, k - 1], ws_asi)
                t_ev[1].record()
                torch.cuda.synchronize()
                asi_ms += t_ev[0].elapsed_time(t_ev[1])
                hist.append(x.k_cur)
                del case, terms
        asi_lk = asi_dev[:, :, 2].double().cpu().tolist()
        table, roles, b_r, b_d, slack = skv.policy_table(asi_lk, cfg.n_drafter * K, b_uni, b_r0, delta, 0)
        cap = max(min(table[l][k - 1], W.c_full(cfg, k)) + cfg.n_tokens(k) for l in range(Lyr) for k in range(1, K + 1))
        calibration = {"pairs": Lyr * K, "queries_per_pair": n_samp, "top_k": top_k, "asi_ms_total": asi_ms,
                       "b_uniform": b_uni, "b_r0": b_r0, "delta": delta, "b_d": b_d, "b_r": b_r, "slack": slack,
                       "drafters_per_scale": [sum(roles[l][k] for l in range(Lyr)) for k in range(K)]}
        log(f"calibration: {Lyr * K} ASI calls {asi_ms:.1f} ms; b_d {b_d}, b_r {b_r}, "
            f"drafters per scale {calibration['drafters_per_scale']}")
        del ws_asi, asi_dev
        torch.cuda.empty_cache()
    bufs = [[(torch.empty(S, H, cap, d, dtype=dtype, device=dev), torch.empty(S, H, cap, d, dtype=dtype, device=dev))
             for _ in range(2)] for _ in range(Lyr)]
    max_q = max(cfg.n_tokens(k) for k in range(1, K + 1))
    ws = torch.empty(skv.workspace_bytes(shape, cap, max_q), dtype=torch.uint8, device=dev)
    out = torch.empty(S, H, max_q, d, dtype=dtype, device=dev)
    outs = {k: out.view(-1)[: U * cfg.n_tokens(k) * d].view(S, H, cfg.n_tokens(k), d) for k in range(1, K + 1)}
    windows = {k: W.window_indices(cfg, cfg.n_tokens(k)) for k in range(1, K + 1)}
    centroids = {k: skv.window_centroids(cfg.sides[k - 1], cfg.sides[k - 1], 4, 4) for k in range(1, K + 1)}
    idx_buf = torch.empty(U * cap, dtype=torch.int32, device=dev)
    log(f"set-up {time.perf_counter() - t_setup:.1f} s")

    events = HipEvents(skv.lib())

    # Marshal the calls once: the cache lengths follow from the budgets, so every argument of
    # every call is known before anything runs.
    variant = args.variant
    stages = STAGES[variant]
    att = stages.index("attend")            # the attend kernel runs between events att and att + 1
    hip = skv.lib()
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    stream_ptr = torch.cuda.current_stream().cuda_stream

    class LibCall:
        """scalekv_step / scalekv_step_append_first; stage events through the library's hook"""
        def __init__(self, prepared):
            self.p = prepared

        def run(self, ev):
            if ev is None:
                self.p(stream_ptr)
            else:
                skv.step_stage_events(ev)
                self.p(stream_ptr)
                skv.step_stage_events(None)

    class PositionalCall:
        """select_positional -> compact -> attend through the single-stage entry points"""
        def __init__(self, x, src, cache_len, n_sink, n_recent, dst, o):
            sink = min(n_sink, cache_len)
            self.keep = sink + min(n_recent, cache_len - sink)
            self.idx = idx_buf.view(-1)[: U * self.keep].view(S, H, self.keep)
            self.a = (x, src, cache_len, n_sink, n_recent, dst, o)

        def run(self, ev):
            x, src, cache_len, n_sink, n_recent, dst, o = self.a
            mark = (lambda i: hip.hipEventRecord(ev[i], stream_ptr) if ev[i] else 0) if ev is not None else (lambda i: 0)
            mark(0)
            skv.select_positional(shape, cache_len, n_sink, n_recent, self.idx)
            mark(1)
            new_len = skv.compact(shape, src[0], src[1], cache_len, self.idx, self.keep, x.k_cur, x.v_cur,
                                  dst[0], dst[1])
            mark(2)
            skv.attend(shape, x.q, dst[0], dst[1], new_len, o)
            mark(3)

    if variant == "pyramid":   # same mean budget per scale as the drafter/refiner table
        table = [[0] * K for _ in range(Lyr)]
        for k in range(1, K + 1):
            full = W.c_full(cfg, k)
            b_uni = full if k < cfg.first_compressed_scale else max(1, int(uniform_frac * full + 0.5))
            for l, b in enumerate(skv.pyramid_budgets(Lyr, b_uni, b_uni // 4 if k >= cfg.first_compressed_scale else b_uni)):
                table[l][k - 1] = b
    def is_big(n_cur):
        """shapes that take the pipelined attention kernel, which also appends the map's K/V itself"""
        return n_cur > 128 and dtype == torch.bfloat16 and d == 128

    calls, meta = [], []
    lens_before_last = None
    lens = [cfg.prefix] * Lyr
    srcs = [prefix[l] for l in range(Lyr)]
    cur_buf = []
    if variant == "literal":
        # read-only start of every pass: the prefix in a buffer with room for the uncompressed scales
        ks = cfg.first_compressed_scale
        room = W.c_full(cfg, min(ks, K)) + cfg.n_tokens(min(ks, K))
        for l in range(Lyr):
            pair = tuple(torch.empty(S, H, room, d, dtype=dtype, device=dev) for _ in range(2))
            pair[0][:, :, :cfg.prefix].copy_(prefix[l][0]); pair[1][:, :, :cfg.prefix].copy_(prefix[l][1])
            cur_buf.append(pair)
    for k in range(1, K + 1):
        n_cur = cfg.n_tokens(k)
        full = W.c_full(cfg, k)
        if k == K:
            lens_before_last = list(lens)
        for l in range(Lyr):
            x = inputs[(l, k)]
            dst = bufs[l][k % 2]
            m = dict(layer=l, scale=k, cache_len=lens[l], n_cur=n_cur, score_bytes=0.0, append_in_attend=0.0)
            append_bytes = 2.0 * 2.0 * n_cur * d * e * U   # K and V, read + write
            if variant in ("scalekv", "pyramid", "calibrated"):
                call = skv.PreparedStep(shape, x.q, x.k_cur, x.v_cur, windows[k], srcs[l][0], srcs[l][1], lens[l],
                                        table[l][k - 1], dst[0], dst[1], outs[k], None, ws)
                keep = call.new_len - n_cur
                m.update(keep=keep, kv_len=keep + n_cur, new_len=call.new_len,
                         move_bytes=2.0 * 2.0 * keep * d * e * U + (4.0 * keep * U if keep < lens[l] else 0)
                         + (0.0 if is_big(n_cur) else append_bytes),
                         append_in_attend=append_bytes if is_big(n_cur) else 0.0)
                if 0 < keep < lens[l]:
                    m["score_bytes"] = (lens[l] * d * e + len(windows[k]) * d * e + 4.0 * lens[l]) * U
                calls.append(LibCall(call))
                srcs[l], lens[l] = dst, call.new_len
            elif variant == "literal":
                # the cache lives in cur_buf[l], which has room for the map; kept rows move to the other buffer
                cur = cur_buf[l]
                dst = bufs[l][1] if cur is bufs[l][0] else bufs[l][0]
                budget = table[l][k - 1] if k >= cfg.first_compressed_scale else full + n_cur
                call = skv.PreparedAppendFirst(shape, x.q, x.k_cur, x.v_cur, centroids[k], args.pool_w, cur[0], cur[1],
                                               lens[l], budget, dst[0], dst[1], outs[k], None, ws)
                assert call.moved == (k >= cfg.first_compressed_scale)
                total = lens[l] + n_cur
                m.update(keep=call.keep, kv_len=total, new_len=call.keep,
                         move_bytes=(0.0 if is_big(n_cur) else append_bytes)
                         + (2.0 * 2.0 * call.keep * d * e * U + 4.0 * call.keep * U if call.moved else 0),
                         append_in_attend=append_bytes if is_big(n_cur) else 0.0)
                calls.append(LibCall(call))
                lens[l] = call.keep
                if call.moved:
                    cur_buf[l] = dst
            else:
                b_uni = full if k < cfg.first_compressed_scale else max(1, int(uniform_frac * full + 0.5))
                n_sink = N_SINK if variant == "sinks" else 0
                call = PositionalCall(x, srcs[l], lens[l], min(n_sink, b_uni), max(0, b_uni - n_sink), dst, outs[k])
                keep = call.keep
                m.update(keep=keep, kv_len=keep + n_cur, new_len=keep + n_cur,
                         move_bytes=2.0 * 2.0 * (keep + n_cur) * d * e * U + 4.0 * keep * U)
                calls.append(call)
                srcs[l], lens[l] = dst, keep + n_cur
            meta.append(m)

    lens_final = list(lens)

    def run_sequence(ev_blocks=None, scale_ev=None):
        """the whole multi-scale sequence: one call per (scale, layer).  scale_ev: K + 1 events,
        recorded on the launch stream before the first call of every scale and after the last call"""
        for i, call in enumerate(calls):
            if scale_ev is not None and i % Lyr == 0:
                hip.hipEventRecord(scale_ev[i // Lyr], stream_ptr)
            call.run(None if ev_blocks is None else ev_blocks[i])
        if scale_ev is not None:
            hip.hipEventRecord(scale_ev[K], stream_ptr)

    n_calls = Lyr * K
    for w in range(args.warmup):
        run_sequence()
        torch.cuda.synchronize()
        log(f"warm-up {w + 1}/{args.warmup} done")

    # Timed region: K passes of the sequence.  The only events inside it bracket launches of the
    # dominant kernel (the pipelined bf16 attention, n_cur > 128); they sit on the launch stream
    # (attached to the kernel's own dispatch) and give that kernel's average duration for the
    # roofline.  Timing every such launch in every pass costs about 1 % of the pass, so each of them
    # is timed in exactly one of the K passes (the j-th such launch of the sequence in pass j mod K).
    n_ev = len(stages) + 1
    big_no = {}
    for i, m in enumerate(meta):
        if is_big(m["n_cur"]):
            big_no[i] = len(big_no)
    ev_steps = [[events.block(n_ev, only=(att, att + 1)) if i in big_no and big_no[i] % args.steps == s else None
                 for i in range(len(meta))] for s in range(args.steps)]
    # one event per scale boundary as well (14 per pass, about 60 us of stream time in all): the
    # per-scale times of the timed passes themselves
    scale_evs = [events.block(K + 1) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_sequence(ev_steps[s], scale_evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    log(f"timed {args.steps} steps: {ms_per_step:.2f} ms per step")

    per_scale_timed = {str(k): sum(events.elapsed_ms(scale_evs[s][k - 1], scale_evs[s][k]) for s in range(args.steps))
                       / args.steps for k in range(1, K + 1)}
    attend_big = dict(ms=0.0, flops=0.0, launches=0, traffic=0.0, min_bytes=0.0)
    attend_by_scale = {}
    traffic_known = (S, H, d) == (16, 16, 128)
    for s in range(args.steps):
        for i, m in enumerate(meta):
            ev = ev_steps[s][i]
            if ev is None:
                continue
            n_cur, kv_len = m["n_cur"], m["kv_len"]
            t_ms = events.elapsed_ms(ev[att], ev[att + 1])
            attend_big["ms"] += t_ms
            attend_big["flops"] += 4.0 * n_cur * kv_len * d * U
            attend_big["launches"] += 1
            bs = attend_by_scale.setdefault(m["scale"], dict(ms=0.0, flops=0.0, launches=0))
            bs["ms"] += t_ms; bs["flops"] += 4.0 * n_cur * kv_len * d * U; bs["launches"] += 1
            attend_big["min_bytes"] += (2.0 * n_cur + 2.0 * kv_len) * d * e * U + m["append_in_attend"]
            if traffic_known and (n_cur, kv_len - n_cur) in ATTEND_PIPE_TRAFFIC:
                attend_big["traffic"] += ATTEND_PIPE_TRAFFIC[(n_cur, kv_len - n_cur)]
            else:
                traffic_known = False

    # ---- one more pass, outside the timed region, with an event at every stage boundary:
    # per-stage and per-scale times and the bandwidth of the two streaming stages
    stage_names = stages
    stage_ms = {n: 0.0 for n in stage_names}
    per_scale_ms = {k: 0.0 for k in range(1, K + 1)}
    per_scale_stage_ms = {k: [0.0] * len(stages) for k in range(1, K + 1)}
    attend_all = dict(ms=0.0, flops=0.0)
    compact_stat = dict(ms=0.0, bytes=0.0)
    compact_last = dict(ms=0.0, bytes=0.0)      # the same at the last (largest) scale only
    score_stat = dict(ms=0.0, bytes=0.0)
    score_last = dict(ms=0.0, bytes=0.0)
    ms_stage_pass = None
    move_slots = [j for j, n in enumerate(stages) if n in ("compact", "append")]
    if not args.no_stage_pass:
        ev_all = [events.block(n_ev) for _ in range(n_calls)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        run_sequence(ev_all)
        torch.cuda.synchronize()
        ms_stage_pass = (time.perf_counter() - t1) * 1e3
        log(f"instrumented pass (events at every stage boundary): {ms_stage_pass:.2f} ms")
        for i, m in enumerate(meta):
            ev, k = ev_all[i], m["scale"]
            t = [events.elapsed_ms(ev[j], ev[j + 1]) for j in range(len(stages))]
            for j, (n, x) in enumerate(zip(stage_names, t)):
                stage_ms[n] += x
                per_scale_stage_ms[k][j] += x
            per_scale_ms[k] += sum(t)
            attend_all["ms"] += t[att]; attend_all["flops"] += 4.0 * m["n_cur"] * m["kv_len"] * d * U
            if m["score_bytes"] > 0 and "score" in stages:
                # a step that ranks: score, select and the gather of the kept rows run in ONE kernel, so the
                # streaming bytes of all three are priced against the time of the three event slots together
                # (where the library ranks in one launch -- bf16, and enough units or a short cache -- the
                # "score" slot brackets exactly that kernel and the other two slots hold nothing but the
                # next event's own cost)
                one_launch = dtype == torch.bfloat16 and m["cache_len"] <= 12288 and (U >= 64 or m["cache_len"] <= 4096)
                t_rank = t[stages.index("score")] if one_launch else \
                    sum(t[stages.index(n)] for n in ("score", "select", "compact"))
                for st_, on in ((compact_stat, True), (compact_last, k == K)):
                    if on:
                        st_["ms"] += t_rank
                        st_["bytes"] += m["score_bytes"] + m["move_bytes"]
                for st_, on in ((score_stat, True), (score_last, k == K)):
                    if on:
                        st_["ms"] += t_rank
                        st_["bytes"] += m["score_bytes"]
            elif "score" not in stages:
                compact_stat["ms"] += sum(t[j] for j in move_slots)
                compact_stat["bytes"] += m["move_bytes"]
                if k == K:
                    compact_last["ms"] += sum(t[j] for j in move_slots)
                    compact_last["bytes"] += m["move_bytes"]
    # ---- the two streaming / matrix kernels on their own, at the last scale's drafter shape, outside
    # the timed region: scalekv_compact doing its whole job (gather + append in one kernel, as the
    # single-stage entry point does) and scalekv_attend over one segment with nothing else to carry
    standalone = None
    if not args.no_stage_pass and variant == "scalekv" and dtype == torch.bfloat16:
        last = max((m for m in meta if m["scale"] == K), key=lambda m: m["keep"])
        l, n_cur, keep, cache_len = last["layer"], last["n_cur"], last["keep"], last["cache_len"]
        x = inputs[(l, K)]
        src = bufs[l][(K - 1) % 2] if K > 1 else prefix[l]
        dst = bufs[l][K % 2]
        idx = torch.stack([torch.sort(torch.randperm(cache_len, device=dev)[:keep])[0] for _ in range(8)])
        idx = idx.repeat((U + 7) // 8, 1)[:U].reshape(S, H, keep).to(torch.int32).contiguous()
        ev = events.block(4)
        reps = 10
        skv.compact(shape, src[0], src[1], cache_len, idx, keep, x.k_cur, x.v_cur, dst[0], dst[1])
        hip.hipEventRecord(ev[0], stream_ptr)
        for _ in range(reps):
            skv.compact(shape, src[0], src[1], cache_len, idx, keep, x.k_cur, x.v_cur, dst[0], dst[1])
        hip.hipEventRecord(ev[1], stream_ptr)
        skv.attend(shape, x.q, dst[0], dst[1], keep + n_cur, outs[K])
        hip.hipEventRecord(ev[2], stream_ptr)
        for _ in range(reps):
            skv.attend(shape, x.q, dst[0], dst[1], keep + n_cur, outs[K])
        hip.hipEventRecord(ev[3], stream_ptr)
        torch.cuda.synchronize()
        c_ms = events.elapsed_ms(ev[0], ev[1]) / reps
        a_ms = events.elapsed_ms(ev[2], ev[3]) / reps
        c_bytes = 2.0 * 2.0 * (keep + n_cur) * d * e * U + 4.0 * keep * U
        a_flops = 4.0 * n_cur * (keep + n_cur) * d * U
        standalone = {
            "shape": f"last scale, drafter: cache_len {cache_len}, keep {keep}, n_cur {n_cur}, {U} units",
            "compact_gather_and_append": {"ms": c_ms, "achieved": c_bytes / (c_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                          "unit": "GB/s", "frac": c_bytes / (c_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "attend_one_segment_no_append": {"ms": a_ms, "achieved": a_flops / (a_ms * 1e-3) / 1e12,
                                             "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                             "frac": a_flops / (a_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        }
        log(f"standalone at the last scale: compact {standalone['compact_gather_and_append']['achieved']:.0f} GB/s, "
            f"attend {standalone['attend_one_segment_no_append']['achieved']:.0f} TFLOP/s")
    events.destroy()
    per_scale_ms = {str(k): v for k, v in per_scale_ms.items()}

    dom = attend_big
    achieved_tflops = dom["flops"] / (dom["ms"] * 1e-3) / 1e12 if dom["ms"] > 0 else 0.0
    roofline = {
        "bound": "mfma", "kernel": "attend_pipe_kernel",
        "achieved": achieved_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": achieved_tflops / PEAK_BF16_TFLOPS,
        "traffic": dom["traffic"] / dom["launches"] if traffic_known and dom["launches"] else None,
        "traffic_unit": "bytes per launch, mean over the timed launches (rocprofv3 FETCH_SIZE/WRITE_SIZE, copy-calibrated)",
        "algorithmic_bytes_per_launch": dom["min_bytes"] / max(1, dom["launches"]),
        "launches": dom["launches"], "avg_launch_ms": dom["ms"] / max(1, dom["launches"]),
        "flops_per_launch_avg": dom["flops"] / max(1, dom["launches"]),
        # the same per scale: every launch of the kernel at that scale, timed once inside the timed region
        "per_scale": {str(k): {"launches": v["launches"], "ms": v["ms"],
                               "achieved": v["flops"] / (v["ms"] * 1e-3) / 1e12 if v["ms"] > 0 else 0.0,
                               "frac": v["flops"] / (v["ms"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if v["ms"] > 0 else 0.0}
                      for k, v in sorted(attend_by_scale.items())},
    }
    gbs = lambda st: st["bytes"] / (st["ms"] * 1e-3) / 1e9 if st["ms"] > 0 else 0.0
    compact_gbs, score_gbs = gbs(compact_stat), gbs(score_stat)

    result = {
        "metric": ("ScaleKV step ms per 1024^2 image batch (13 scales)" if cfg.name == "2b_1024"
                   else f"ScaleKV step ms per image batch ({cfg.name})")
                  + ("" if variant == "scalekv" else f" [variant: {variant}]"),
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {S} sequences x {H} heads x d{d}, {Lyr} layers, {K} scales "
                               f"({cfg.image_tokens} image tokens, {cfg.prefix}-token prefix), "
                               f"{cfg.n_drafter} drafters at {cfg.drafter_frac:.0%} / {Lyr - cfg.n_drafter} refiners at "
                               f"{cfg.refiner_frac:.0%} per scale, window {cfg.window}",
                   "variant": variant, "calls_per_step": n_calls, "shared_inputs": bool(args.shared_inputs)},
        "roofline": roofline,
        "per_scale_ms": per_scale_timed,
        "parity": None,
        "stage_pass": None if ms_stage_pass is None else {
            "note": "one extra pass outside the timed region with an event at every stage boundary",
            "stages": list(stages),
            "ms": ms_stage_pass, "stage_ms": stage_ms, "per_scale_ms": per_scale_ms,
            "per_scale_stage_ms": {str(k): [round(x, 4) for x in v] for k, v in per_scale_stage_ms.items()}},
        "standalone_kernels": standalone,
        "calibration": calibration,
        "hip_graph_replay": None,
        "attend_clock": None,
        "attend_tflops_all_scales": attend_all["flops"] / (attend_all["ms"] * 1e-3) / 1e12 if attend_all["ms"] else 0.0,
        "compact_hbm": {"achieved": compact_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": compact_gbs / PEAK_HBM_GBS,
                        "last_scale": gbs(compact_last), "last_scale_frac": gbs(compact_last) / PEAK_HBM_GBS,
                        "kernel": "select_kernel<true, true, 128, 4>: score + select + gather of the kept rows in one launch",
                        "note": "algorithmic bytes of the kernel that carries the compaction (keys read once for the "
                                "score, kept K/V rows read and written) over its time in the instrumented pass, steps "
                                "that rank only; its fp32 logits (64 B per key, mostly L2) are not counted; the map's "
                                "K/V are appended by the attention kernel and counted there"},
        "score_hbm": {"achieved": score_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": score_gbs / PEAK_HBM_GBS,
                      "last_scale": gbs(score_last), "last_scale_frac": gbs(score_last) / PEAK_HBM_GBS,
                      "note": "the score's own bytes (keys once) over the time of the same one kernel, which also selects and gathers"},
    }
    # ---- context, not targets: KV-cache bytes of this workload with and without eviction (the
    # quantity the paper reports), the paper's own numbers, and what the vendor libraries reach on
    # this very box (a large bf16 GEMM, a large device-to-device copy) next to the published peaks
    row_gb = 2.0 * d * e * U / 1e9     # K and V bytes of one cache row over all units of a layer
    hist_full = W.c_full(cfg, K) * row_gb * Lyr
    hist_kept = sum(m["keep"] for m in meta if m["scale"] == K) * row_gb
    result["kv_cache_gb"] = {
        "history_before_last_scale_full": hist_full, "history_before_last_scale_kept": hist_kept,
        "kept_fraction": hist_kept / hist_full,
        "after_last_scale_full": (W.c_full(cfg, K) + cfg.n_tokens(K)) * row_gb * Lyr,
        "after_last_scale_held": sum(lens_final) * row_gb,
        "note": "history = every row cached before the last scale; the last map's own rows are appended unpruned"}
    result["paper_context"] = {
        "kv_cache_gb_infinity_8b_batch8_1024": {"full": 85.0, "scalekv_10pct": 8.5},
        "speedup": "up to 1.25x end to end on one NVIDIA H20 (whole model, not this path alone)",
        "note": "the paper's numbers, other hardware, memory hardware not stated: context only"}
    if not args.no_stage_pass:
        n = 8192
        a = torch.randn(n, n, device=dev, dtype=torch.bfloat16); b = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev); dstb = torch.empty_like(src)
        # long enough to be past the library's and the clock's warm-up: a handful of calls reads
        # 20 % low (1.1 against 1.38 PFLOP/s sustained on the same box)
        n_gemm, n_copy = 100, 20
        for _ in range(20):
            torch.matmul(a, b)
        dstb.copy_(src)
        t_ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        t_ev[0].record()
        for _ in range(n_gemm):
            torch.matmul(a, b)
        t_ev[1].record()
        for _ in range(n_copy):
            dstb.copy_(src)
        t_ev[2].record()
        torch.cuda.synchronize()
        gemm_tflops = n_gemm * 2.0 * n ** 3 / (t_ev[0].elapsed_time(t_ev[1]) * 1e-3) / 1e12
        copy_gbs = n_copy * 2.0 * (1 << 30) / (t_ev[1].elapsed_time(t_ev[2]) * 1e-3) / 1e9
        result["same_box_references"] = {
            "bf16_gemm_8192_tflops": gemm_tflops, "copy_1gib_gbs": copy_gbs,
            "attend_vs_gemm": roofline["achieved"] / gemm_tflops if gemm_tflops else None,
            "note": "torch.matmul (vendor GEMM library, 100 calls after 20 of warm-up) and torch copy on this box, "
                    "outside the timed region"}
        del a, b, src, dstb
        log(f"same box: bf16 GEMM {gemm_tflops:.0f} TFLOP/s, copy {copy_gbs:.0f} GB/s")
    # ---- parity of what was just timed: sampled units of the last scale through the oracle
    if not args.no_parity and variant == "scalekv":
        log("replaying sampled last-scale units through the CPU oracle ...")
        result["parity"] = parity_replay(torch, skv, W, cfg, shape, inputs, prefix, bufs, table, lens_before_last,
                                         windows, ws)
        log(f"parity: {result['parity']}")
    # ---- the same sequence captured once into a HIP graph and replayed (what a serving loop with
    # fixed shapes would do); reported beside the eager number, never in place of it.  Last GPU
    # work of the run, so that a failed capture cannot disturb any other measurement.
    if not args.no_graph_pass and variant in ("scalekv", "pyramid", "literal", "calibrated"):
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                sp = torch.cuda.current_stream().cuda_stream
                for call in calls:
                    call.p(sp)
            graph.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            result["hip_graph_replay"] = {"ms_per_step": (time.perf_counter() - t1) * 1e3 / args.steps,
                                          "replays": args.steps, "calls_captured": n_calls}
            log(f"graph replay: {result['hip_graph_replay']['ms_per_step']:.2f} ms per step")
            del graph
        except Exception as exc:   # the eager numbers above stand on their own
            result["hip_graph_replay"] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
            log(f"graph replay failed: {exc}")
    if not args.no_clock_leg and variant == "scalekv":
        result["attend_clock"] = attend_clock_leg()
        log(f"attention kernel's clock: {result['attend_clock']}")
    if not args.no_cpu_baseline and variant == "scalekv":
        log("timing the CPU oracle on its sample ...")
        del inputs, bufs
        torch.cuda.empty_cache()
        result["cpu_baseline"] = cpu_baseline(cfg, W)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
