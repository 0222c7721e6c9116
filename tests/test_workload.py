"""Input generator: determinism, distribution, and the structure the workloads promise."""
import numpy as np
import torch

from workload import workload, gen_weights, gen_prompt, weight_specs, WORKLOAD_NAMES, EXTRA_WORKLOAD_NAMES
from workload.gen import gen_normal_bf16, gen_tensor


def test_counter_based_and_chunk_independent():
    a = gen_normal_bf16(0, "t", 10007, 0.02, chunk=1 << 26)
    b = gen_normal_bf16(0, "t", 10007, 0.02, chunk=4096)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    c = gen_normal_bf16(1, "t", 10007, 0.02)
    assert not torch.equal(a.view(torch.int16), c.view(torch.int16))
    d = gen_normal_bf16(0, "u", 10007, 0.02)
    assert not torch.equal(a.view(torch.int16), d.view(torch.int16))


def test_normal_moments():
    x = gen_normal_bf16(0, "moments", 1 << 20, 0.02).double()
    assert abs(x.mean().item()) < 1e-4
    assert abs(x.std().item() - 0.02) < 2e-4
    z = x / 0.02
    assert abs((z ** 4).mean().item() - 3.0) < 0.05          # kurtosis of a normal
    assert abs((z.abs() < 1).double().mean().item() - 0.6827) < 5e-3


def test_tiny_weights_and_lm_head_scale():
    w = workload("tiny")
    ws = dict(gen_weights(w.model, 0))
    assert set(ws) == {n for n, _, _ in weight_specs(w.model)}
    assert abs(ws["lm_head"].float().std().item() - 0.5) < 0.01
    assert abs(ws["l1.w_down"].float().std().item() - 0.02) < 0.001
    assert torch.all(ws["final_norm"].float() == 1)
    assert ws["l0.w_gate"].shape == (688, 256)


def test_lm_head_scale_rule():
    for name in ("llada", "dream"):
        m = workload(name).model
        assert abs(m.lm_head_std * m.d_model ** 0.5 - 8.0) < 1e-9


def test_prompts_exclude_mask_and_lengths():
    for name in WORKLOAD_NAMES + EXTRA_WORKLOAD_NAMES:
        w = workload(name)
        for r, lp in enumerate(w.prompt_lens):
            p = gen_prompt(w.model, w.seed, r, lp)
            assert p.shape == (lp,) and p.min() >= 0 and p.max() < w.model.mask_id
    x16 = workload("llada_x16")
    assert x16.n_requests == 16 and min(x16.prompt_lens) >= 256 and max(x16.prompt_lens) <= 1024
    assert sum(workload("llada").block_sizes) == 120


def test_dream_has_bias_tensors():
    names = [n for n, _, _ in weight_specs(workload("dream").model)]
    assert "l0.bq" in names and "l27.bv" in names
    assert "l0.bq" not in [n for n, _, _ in weight_specs(workload("llada").model)]
