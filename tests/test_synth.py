"""The seeded input generator: determinism, slice consistency, distribution."""
import numpy as np
import torch

import synth


def test_deterministic_and_slice_consistent():
    a = synth.hash_normal(7, 3, (1000, 37), 0.02, torch.float32)
    b = synth.hash_normal(7, 3, (1000, 37), 0.02, torch.float32)
    assert torch.equal(a, b)
    # a longer tensor with the same stream starts with the same values
    c = synth.hash_normal(7, 3, (2000, 37), 0.02, torch.float32)
    assert torch.equal(c[:1000], a)
    assert not torch.equal(a, synth.hash_normal(8, 3, (1000, 37), 0.02, torch.float32))
    assert not torch.equal(a, synth.hash_normal(7, 4, (1000, 37), 0.02, torch.float32))


def test_distribution():
    x = synth.hash_normal(1, 5, (400000,), 0.02, torch.float32).double().numpy()
    assert abs(x.mean()) < 2e-4 and abs(x.std() - 0.02) < 2e-4
    assert abs(np.mean(np.abs(x) < 0.02) - 0.6827) < 0.01
    b = synth.hash_normal(1, 5, (400000,), 0.02, torch.bfloat16)
    assert torch.equal(b, torch.from_numpy(x).float().to(torch.bfloat16))
    u = synth.hash_uniform(1, 6, 200000).numpy()
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 0.005
    t = synth.hash_tokens(1, 7, 200000, 1000).numpy()
    assert t.min() >= 0 and t.max() < 1000
    assert np.bincount(t, minlength=1000).min() > 120


def test_presets():
    c3 = synth.CONFIGS["c3_70b"]
    assert c3.M == 36 and c3.q_dim == 8192 and c3.kv_dim == 1024 and c3.group == 8
    per_layer = sum(a * b for a, b in synth.layer_weight_shapes(c3).values())
    assert per_layer == 855_638_016                       # parameters per 70B layer
    c1 = synth.CONFIGS["c1_tiny"]
    assert sum(a * b for a, b in synth.layer_weight_shapes(c1).values()) == 724_992
    temps = synth.make_row_temperature(c1)
    assert temps.shape == (1, 5) and set(np.round(temps.double().numpy().ravel(), 4)) <= {0.3, 1.0, 3.0}
    c5 = synth.CONFIGS["c5_stress"]
    t5 = synth.make_row_temperature(c5).numpy()
    assert t5.min() >= 0.1 - 1e-6 and t5.max() <= 10 + 1e-5 and t5.shape == (64, 17)
    k, v = synth.make_kv_prefix(c1, 0)
    assert k.shape == (1, 128, 2, 64) and abs(k.double().std().item() - 1) < 0.02
