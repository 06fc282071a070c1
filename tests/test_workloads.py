"""The seeded generator: slices regenerate the same bits, shapes and moments
are what the workload statements say."""
import pytest
import torch

import workloads as W


def test_unit_slices_equal_full_tensor():
    cfg = W.get_config("2b_512")
    full = W.make_step_inputs(cfg, 3, 6)
    part = W.make_step_inputs(cfg, 3, 6, units=[5, 11])
    assert full.q.shape == (1, 16, 144, 128) and full.q.dtype == torch.bfloat16
    for name in ("q", "k_cur", "v_cur"):
        f, p = getattr(full, name), getattr(part, name)
        assert torch.equal(f[0, 5], p[0]) and torch.equal(f[0, 11], p[1])
    kf, vf = W.make_prefix(cfg, 2)
    kp, vp = W.make_prefix(cfg, 2, units=[9])
    assert torch.equal(kf[0, 9], kp[0]) and torch.equal(vf[0, 9], vp[0])


def test_streams_differ_by_layer_scale_and_tensor():
    cfg = W.get_config("2b_512")
    a = W.make_step_inputs(cfg, 0, 5, units=[0])
    b = W.make_step_inputs(cfg, 1, 5, units=[0])
    c = W.make_step_inputs(cfg, 0, 5, units=[1])
    assert not torch.equal(a.q, b.q) and not torch.equal(a.q, c.q)
    assert not torch.equal(a.q, a.k_cur) and not torch.equal(a.k_cur, a.v_cur)


def test_moments():
    g = W.normal_tensor(W.stream_key(0, 77), (400000,))
    assert abs(float(g.mean())) < 0.01 and abs(float(g.std()) - 1.0) < 0.01
    cfg = W.get_config("2b_512")
    x = W.make_step_inputs(cfg, 0, 9, units=[0, 1])
    logits = x.q[0].float() @ x.k_cur[0].float().T / 128 ** 0.5
    assert 3.0 < float(logits.std()) < 5.5     # peaked attention
    tiny = W.make_step_inputs(W.get_config("tiny"), 0, 4)
    assert tiny.q.dtype == torch.float32 and tiny.q.shape == (1, 2, 64, 64)
    assert abs(float(tiny.q.std()) - 0.125) < 0.01


def test_final_scale_case_has_dominant_keys():
    cfg = W.get_config("final_scale")
    fc = W.make_final_scale_case(cfg, units=[0, 7], n_q=32, hist_len=3000)
    frac = float(fc.boosted.float().mean())
    assert 0.005 < frac < 0.02
    logits = fc.q[0].float() @ fc.k_hist[0].float().T / 128 ** 0.5
    gap = logits[:, fc.boosted[0]].mean() - logits[:, ~fc.boosted[0]].mean()
    assert 3.5 < float(gap) < 4.5
    assert W.final_scale_budgets(cfg) == [324, 649, 1298, 6489]


@pytest.mark.gpu
def test_generator_is_device_independent():
    for name, layer, scale in (("2b_512", 1, 7), ("8b_1024", 2, 5), ("tiny", 1, 4)):
        cfg = W.get_config(name)
        units = [0, 3]
        a = W.make_step_inputs(cfg, layer, scale, "cpu", units)
        b = W.make_step_inputs(cfg, layer, scale, "cuda", units)
        for n in ("q", "k_cur", "v_cur"):
            assert torch.equal(getattr(a, n), getattr(b, n).cpu()), (name, n)
    cfg = W.get_config("final_scale")
    a = W.make_final_scale_case(cfg, "cpu", [1], 64, 700)
    b = W.make_final_scale_case(cfg, "cuda", [1], 64, 700)
    assert torch.equal(a.q, b.q.cpu()) and torch.equal(a.k_hist, b.k_hist.cpu())
