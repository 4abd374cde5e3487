"""The input generators: storage rounding against a library conversion, and the structure
of the synthetic traces and placements."""
import numpy as np
import torch

import synth_inputs as syn


def test_bf16_rounding_matches_library_conversion():
    a = syn.rng(1).standard_normal(100000, dtype=np.float32) * np.float32(3.0)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]  # exact ties: round to even
    bits = syn.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    np.testing.assert_array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    np.testing.assert_array_equal(syn.bf16_bits_to_f32(bits), ref.float().numpy())
    q = syn.quantize(a, "bf16")
    np.testing.assert_array_equal(syn.quantize(q, "bf16"), q)


def test_trace_and_placement_structure():
    trace, perms = syn.planted_trace(6, 50000, 16, 0.7, seed=2)
    assert trace.dtype == np.int32 and trace.min() >= 0 and trace.max() < 16
    for l in range(5):
        follow = (perms[l][trace[l]] == trace[l + 1]).mean()
        assert abs(follow - (0.7 + 0.3 / 16)) < 0.01
    pl = syn.balanced_random_placement(6, 16, 4, seed=3)
    for l in range(6):
        assert (np.bincount(pl[l], minlength=4) == 4).all()
    z, _ = syn.planted_trace(2, 200000, 32, 0.7, seed=4, marginal="zipf")
    loads = np.sort(np.bincount(z[0], minlength=32))[::-1] / 200000
    assert abs(loads[0] - syn.zipf_loads(32, 1.1)[0]) < 0.01
    assert loads[0] > 10 * loads[-1]
    idx, em = syn.local_routing(syn.CONFIGS[4], seed=5)
    assert (em[idx] >= 0).all() and (em >= 0).sum() == 8


def test_generators_are_deterministic():
    c = syn.CONFIGS[1]
    np.testing.assert_array_equal(syn.tokens(c), syn.tokens(c))
    w1a, w2a = syn.expert_weights(c)
    w1b, w2b = syn.expert_weights(c)
    np.testing.assert_array_equal(w1a, w1b)
    assert w1a.shape == (8, 256, 64) and w2a.shape == (8, 64, 256)
    assert abs(w1a.std() - 0.02) < 1e-3
