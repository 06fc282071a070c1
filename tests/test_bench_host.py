"""Host-side checks of bench.py that need no GPU: the one-GPU contract of its command line and
that its table of measured attention-kernel traffic covers every shape the headline workload
launches (a stale table would silently turn `roofline.traffic` into null)."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be mistaken for a result


def test_traffic_table_covers_every_pipelined_shape_of_the_headline_workload():
    bench = _bench_module()
    cfg = W.get_config("2b_1024")
    table = W.budget_table(cfg)
    lens = [cfg.prefix] * cfg.n_layer
    seen = set()
    for k in range(1, cfg.n_scale + 1):
        n_cur = cfg.n_tokens(k)
        for l in range(cfg.n_layer):
            keep = min(table[l][k - 1], lens[l])
            if n_cur > 128:
                seen.add((n_cur, keep))
            lens[l] = keep + n_cur
    assert seen, "the workload should have shapes that take the pipelined kernel"
    missing = sorted(seen - set(bench.ATTEND_PIPE_TRAFFIC))
    assert not missing, f"no measured traffic for shapes {missing}"


def test_stage_lists_match_the_event_slots_of_the_library_hook():
    bench = _bench_module()
    for variant in bench.VARIANTS:
        stages = bench.STAGES[variant]
        assert "attend" in stages
        assert len(stages) + 1 <= 5       # the step hook marks at most five boundaries


def test_timeline_summary_reads_per_xcd_times_from_the_records():
    """Synthetic records of a 2-round launch on 8 XCDs x 2 compute units x 2 slots: XCD x's
    workgroups last 100 + 10 x us, so the launch ends with XCD 7 and the others idle before that."""
    import ctypes

    import numpy as np
    bench = _bench_module()
    n_wg, t0 = 64, 5_000_000
    rec = np.zeros((n_wg, 7), dtype=np.uint64)
    for wg in range(n_wg):
        x, local = wg % 8, wg // 8              # 8 workgroups per XCD: 4 slots, 2 rounds
        dur = 100 + 10 * x
        start = (local // 4) * dur
        cu = (local % 4) // 2
        rec[wg] = [t0 + 100 * start, t0 + 100 * (start + 3), t0 + 100 * (start + dur - 2), t0 + 100 * (start + dur),
                   cu << 8, 1000, 1000 + 2000 * dur]  # 10 ns ticks; compute unit in bits 8-11; a 2000 MHz clock counter

    class FakeLib:
        @staticmethod
        def scalekv_timeline_read(dst, n):
            ctypes.memmove(dst, rec.ctypes.data, rec.nbytes)
            return 0

    class FakeBinding:
        @staticmethod
        def lib():
            return FakeLib

    s = bench.timeline_summary(FakeBinding, n_wg)
    assert s["workgroups"] == 64 and s["compute_units"] == 16
    assert s["span_us"] == 340.0                                   # XCD 7: two rounds of 170 us
    assert [p["last_end_us"] for p in s["per_xcd"]] == [200.0 + 20 * x for x in range(8)]
    assert [p["mean_wg_us"] for p in s["per_xcd"]] == [100.0 + 10 * x for x in range(8)]
    assert [p["clock_counter_mhz"] for p in s["per_xcd"]] == [2000.0] * 8
    assert s["start_to_first_tile_us"] == 3.0 and s["loop_end_to_end_us"] == 2.0
    assert abs(s["idle_at_the_end"] - (1 - 270.0 / 340.0)) < 1e-3  # mean end over the XCDs is 270 us
