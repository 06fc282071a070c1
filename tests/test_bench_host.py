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
