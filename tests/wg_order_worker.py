"""Runs a fixed list of library calls on seeded inputs and returns (or saves) every output.

tests/test_gpu_wg_order.py runs it twice: in the test process with the library in the tree, and in
a child process whose SCALEKV_LIBRARY names the build that walks every grid backwards
(python -m paper_2505_19602_amd.build --variant reversed_order).  Not collected by pytest."""
import os
import sys

import numpy as np
import torch

DEV = "cuda"


def run_all():
    import paper_2505_19602_amd as skv
    import workloads as W

    out = {"library": np.array(os.path.basename(skv.lib_path()))}

    def rand(key, shape, dtype):
        return W.normal_tensor(W.stream_key(4321, key), shape).to(dtype).to(DEV)

    def keep_np(name, t):
        t = t.detach().cpu()
        out[name] = (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).numpy().copy()

    # (tag, S, H, d, n_cur, cache_len, budget, dtype): pipelined attention with a fused ranking
    # kernel, the small-map attention kernel, a head size of 64, fp32, and a cache longer than the
    # ranking kernel's LDS (the two-launch route)
    cases = [("pipe", 3, 5, 128, 300, 900, 333, torch.bfloat16),
             ("pipe_ragged", 2, 4, 128, 400, 1500, 210, torch.bfloat16),
             ("small", 2, 3, 128, 36, 140, 50, torch.bfloat16),
             ("d64", 2, 2, 64, 70, 260, 90, torch.bfloat16),
             ("fp32", 1, 2, 64, 33, 150, 60, torch.float32),
             ("long", 1, 2, 128, 130, 12600, 1000, torch.bfloat16)]
    for c, (tag, S, H, d, n_cur, L, budget, dtype) in enumerate(cases):
        print(f"workgroup order: step {tag}: {S}x{H} units, {n_cur} queries, {L} cached rows", flush=True)
        shape = skv.Shape(S, H, d, dtype)
        q, kc, vc = (rand(10 * c + i, (S, H, n_cur, d), dtype) for i in range(3))
        ks, vs = rand(10 * c + 3, (S, H, L, d), dtype), rand(10 * c + 4, (S, H, L, d), dtype)
        win = list(range(max(0, n_cur - 16), n_cur))
        keep = min(budget, L)
        ws = torch.zeros(skv.workspace_bytes(shape, L, n_cur), dtype=torch.uint8, device=DEV)
        kd = torch.zeros((S, H, keep + n_cur, d), dtype=dtype, device=DEV); vd = torch.zeros_like(kd)
        o = torch.zeros((S, H, n_cur, d), dtype=dtype, device=DEV)
        idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        skv.step(shape, q, kc, vc, win, ks, vs, L, budget, kd, vd, o, idx, ws)
        torch.cuda.synchronize()
        for name, t in (("k_dst", kd), ("v_dst", vd), ("out", o), ("idx", idx)):
            keep_np(f"step_{tag}_{name}", t)

        # the single stages on the same inputs
        scores = torch.zeros((S, H, L), dtype=torch.float32, device=DEV)
        skv.score(shape, q[:, :, -len(win):].contiguous(), ks, L, scores, ws)
        idx2 = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
        skv.select(shape, scores, L, budget, idx2)
        kd2 = torch.zeros((S, H, keep + n_cur, d), dtype=dtype, device=DEV); vd2 = torch.zeros_like(kd2)
        skv.compact(shape, ks, vs, L, idx2, keep, kc, vc, kd2, vd2)
        o2 = torch.zeros_like(o)
        skv.attend(shape, q, kd2, vd2, keep + n_cur, o2)
        torch.cuda.synchronize()
        for name, t in (("scores", scores), ("idx", idx2), ("k_dst", kd2), ("v_dst", vd2), ("out", o2)):
            keep_np(f"stages_{tag}_{name}", t)

    # the literal order of Sec. 3.3 (append, attend, rank with pooling and forced window rows)
    print("workgroup order: step_append_first", flush=True)
    S, H, d, n_cur, L, budget, dtype = 2, 3, 128, 144, 500, 120, torch.bfloat16
    shape = skv.Shape(S, H, d, dtype)
    q, kc, vc = (rand(900 + i, (S, H, n_cur, d), dtype) for i in range(3))
    cap = L + n_cur
    kcache, vcache = rand(903, (S, H, cap, d), dtype), rand(904, (S, H, cap, d), dtype)
    win = skv.window_centroids(12, 12)
    keep = len(win) + min(budget, L + n_cur - len(win))
    kn = torch.zeros((S, H, keep, d), dtype=dtype, device=DEV); vn = torch.zeros_like(kn)
    o = torch.zeros((S, H, n_cur, d), dtype=dtype, device=DEV)
    idx = torch.full((S, H, keep), -1, dtype=torch.int32, device=DEV)
    ws = torch.zeros(skv.workspace_bytes(shape, cap, n_cur), dtype=torch.uint8, device=DEV)
    skv.step_append_first(shape, q, kc, vc, win, 7, kcache, vcache, L, budget, kn, vn, o, idx, ws)
    torch.cuda.synchronize()
    for name, t in (("k_next", kn), ("v_next", vn), ("out", o), ("idx", idx)):
        keep_np(f"literal_{name}", t)

    # Eq. 2 terms and position-only retention
    print("workgroup order: asi, select_positional", flush=True)
    S, H, d, dtype = 2, 2, 128, torch.bfloat16
    shape = skv.Shape(S, H, d, dtype)
    hist, cur = 700, 256
    k = rand(950, (S, H, hist + cur, d), dtype)
    qs = rand(951, (S, H, 16, d), dtype)
    ws = torch.zeros(skv.workspace_bytes(shape, hist + cur, 16), dtype=torch.uint8, device=DEV)
    terms = torch.zeros((S, H, 16, 2), dtype=torch.float32, device=DEV)
    asi_out = torch.zeros(3, dtype=torch.float32, device=DEV)
    skv.asi(shape, qs, k, hist, cur, 64, terms, asi_out, ws)
    torch.cuda.synchronize()
    keep_np("asi_terms", terms)
    keep_np("asi_out", asi_out)
    idxp = torch.full((S, H, 80), -1, dtype=torch.int32, device=DEV)
    skv.select_positional(shape, 500, 16, 64, idxp)
    torch.cuda.synchronize()
    keep_np("positional_idx", idxp)
    return out


if __name__ == "__main__":
    np.savez(sys.argv[1], **run_all())
    print("workgroup order: worker done", flush=True)
