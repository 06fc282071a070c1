"""Run a few scalekv_step calls of one shape, for use under rocprofv3.

    python3 -m paper_2505_19602_amd.profile_step --cache-len 3350 --budget 1622 --n-cur 4096
    python3 -m paper_2505_19602_amd.profile_step --case 3350,1622,4096 --case 2513,324,4096

Each --case is cache_len,budget,n_cur; the cases run in the order given, so the
n-th group of the library's kernels in the trace belongs to the n-th case.

A 1 GiB device-to-device copy is issued first: the hardware byte counters
(FETCH_SIZE, WRITE_SIZE) are calibrated against its known size.
"""
from __future__ import annotations

import argparse

import torch

from . import Shape, step, workspace_bytes


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n-seq", type=int, default=16)
    ap.add_argument("--n-head", type=int, default=16)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--cache-len", type=int, default=3350)
    ap.add_argument("--budget", type=int, default=1622)
    ap.add_argument("--n-cur", type=int, default=4096)
    ap.add_argument("--case", action="append", default=[],
                    help="cache_len,budget,n_cur (repeatable; overrides the three single options)")
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    dev, dt = "cuda", torch.bfloat16
    S, H, d = a.n_seq, a.n_head, a.head_dim
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    shape = Shape(S, H, d, dt)
    g = torch.Generator(device=dev).manual_seed(0)
    rnd = lambda rows: torch.randn(S, H, rows, d, device=dev, dtype=torch.float32, generator=g).to(dt)
    cases = [tuple(int(x) for x in c.split(",")) for c in a.case] or [(a.cache_len, a.budget, a.n_cur)]
    for (L, budget, n) in cases:
        q, kc, vc, ks, vs = rnd(n), rnd(n), rnd(n), rnd(L), rnd(L)
        keep = min(budget, L)
        kd = torch.empty(S, H, keep + n, d, device=dev, dtype=dt)
        vd = torch.empty_like(kd)
        out = torch.empty_like(q)
        ws = torch.empty(workspace_bytes(shape, L, n), dtype=torch.uint8, device=dev)
        win = list(range(max(0, n - 16), n))
        for _ in range(a.reps):
            step(shape, q, kc, vc, win, ks, vs, L, budget, kd, vd, out, None, ws)
        torch.cuda.synchronize()
        print(f"ran {a.reps} steps: cache_len={L} keep={keep} n_cur={n} units={S * H}", flush=True)
        del q, kc, vc, ks, vs, kd, vd, out, ws


if __name__ == "__main__":
    main()
