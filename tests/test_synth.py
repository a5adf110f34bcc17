"""The seeded generators: determinism, slab/full-volume consistency, distribution sanity, bf16 rounding."""
import numpy as np
import pytest

import synth


def test_slab_is_a_cut_of_the_full_volume_and_zero_outside():
    full = synth.slab("normal", 7, 3, (2, 3, 8, 4, 5), 0, 8)
    s = synth.slab("normal", 7, 3, (2, 3, 8, 4, 5), 3, 10)
    assert np.array_equal(s[:, :, :5], full[:, :, 3:8]) and not s[:, :, 5:].any()
    assert np.array_equal(full.ravel(), synth.flat("normal", 7, 3, (2 * 3 * 8 * 4 * 5,)))
    assert not np.array_equal(full, synth.slab("normal", 8, 3, (2, 3, 8, 4, 5), 0, 8))
    assert not np.array_equal(full, synth.slab("normal", 7, 4, (2, 3, 8, 4, 5), 0, 8))


def test_distributions():
    u = synth.flat("uniform", 1, 1, (200000,), -1.0, 1.0)
    assert u.min() > -1 and u.max() < 1 and abs(u.mean()) < 0.01 and abs(u.var() - 1 / 3) < 0.01
    g = synth.flat("normal", 1, 2, (200000,))
    assert abs(g.mean()) < 0.01 and abs(g.var() - 1) < 0.02
    c = synth.flat("cosmo", 1, 3, (200000,))
    k = np.expm1(c)
    assert c.min() == 0 and np.allclose(k, np.round(k)) and 1.3 < k.mean() < 2.0 and (k == 0).mean() > 0.3


def test_bf16_rounding_is_nearest_even():
    torch = pytest.importorskip("torch")
    a = np.concatenate([synth.flat("normal", 3, 1, (50000,)) * 100, [1.0, 1.00390625, 1.01171875, 0.0, -0.0]]).astype(np.float32)
    ours = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(ours), torch.from_numpy(a).to(torch.bfloat16).float().numpy())
