"""The seeded input generators: determinism, slice-independence, distribution shape, workload sizes."""
import numpy as np
import torch

import synth


def test_workload_sizes():
    want = {"tiny": 1_048_576, "gpt2s": 124_439_808, "gpt1p3b": 1_315_723_264, "llama7b": 6_738_415_616,
            "llama7b_w1": 6_738_415_616}
    for k, p in want.items():
        assert synth.get_workload(k).num_params == p
    w = synth.get_workload("ragged7b")
    assert len(w.tensors) == 2000
    sizes = [t.numel for t in w.tensors]
    assert min(sizes) >= 64 and max(sizes) == 131_072_000
    extras = [t for t in w.tensors if t.name.startswith("x")]
    assert len(extras) == 1709 and all(t.numel % 128 for t in extras)
    flags = [t.weight_decay for t in w.tensors]
    assert 0.4 < sum(flags) / len(flags) < 0.6
    assert [t.numel for t in synth.get_workload("ragged7b").tensors] == sizes      # deterministic


def test_counter_based_slices_agree():
    idx = torch.arange(0, 5000, dtype=torch.int64)
    full = synth.grad_values(7, 3, 2, idx, "normal", 1e-3, "bf16")
    part = synth.grad_values(7, 3, 2, idx[1234:2345], "normal", 1e-3, "bf16")
    assert torch.equal(full[1234:2345], part)
    other = synth.grad_values(7, 3, 1, idx, "normal", 1e-3, "bf16")
    assert not torch.equal(full, other)
    per = synth.grad_values(7, 3, 2, idx, "normal", 1e-3, "f32", period=1009)
    base = synth.grad_values(7, 3, 2, idx[:1009], "normal", 1e-3, "f32")
    assert torch.equal(per[1009:2018], base) and torch.equal(per[:1009], base)


def test_distributions():
    idx = torch.arange(0, 400_000, dtype=torch.int64)
    g = synth.grad_values(1, 1, 0, idx, "normal", 1e-3, "f32").double()
    assert abs(g.mean().item()) < 1e-5 and abs(g.std().item() / 1e-3 - 1) < 0.01
    kurt = ((g / g.std()) ** 4).mean().item()
    assert 2.5 < kurt < 3.1
    t = synth.grad_values(1, 1, 0, idx, "t3", 1e-3, "f32").double()
    assert (t.abs() > 6e-3).float().mean().item() > 0.004      # heavy tails: P(|t3| > 6) ~ 0.0093
    assert (g.abs() > 6e-3).sum().item() == 0
    p = synth.param_values(1, idx).double()
    assert abs(p.std().item() / 0.02 - 1) < 0.01


def test_bf16_rounding_matches_library():
    x = torch.randn(100_000) * 1e-3
    bits = synth.f32_to_bf16_bits(x)
    assert torch.equal(bits.view(torch.bfloat16), x.to(torch.bfloat16))


def test_arrival_order_is_a_permutation():
    for step in (1, 2, 3):
        o = synth.arrival_order(5, step, 257)
        assert sorted(o) == list(range(257))
    assert synth.arrival_order(5, 1, 257) != synth.arrival_order(5, 2, 257)
    assert synth.arrival_order(5, 1, 257) == synth.arrival_order(5, 1, 257)
