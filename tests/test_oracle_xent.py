"""Pins for the oracle's per-voxel softmax cross-entropy (no GPU): a library routine (torch CPU float64 cross_entropy with
autograd), closed forms (equal logits give log C and a gradient of (1/C - onehot)/count; a huge margin gives 0), invariance
under a per-voxel shift of all logits, gradients summing to zero over the classes, central differences, and additivity
over depth shards with the halo planes ignored."""
import numpy as np
import pytest
import torch

import oracle as orc
from oracle import Slab

RNG = np.random.default_rng(2007_12856 + 9)


def case(n=2, c=3, d=4, h=3, w=5):
    return RNG.normal(0, 2.0, size=(n, c, d, h, w)), RNG.integers(0, c, size=(n, d, h, w))


@pytest.mark.parametrize("c", [2, 3, 5])
def test_matches_torch_float64(c):
    z, lab = case(c=c)
    loss, dz = orc.softmax_xent_fwd_bwd(Slab(z), lab)
    zt = torch.tensor(z, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(lab), reduction="mean")
    lt.backward()
    assert abs(loss - lt.item()) <= 1e-12 * abs(lt.item())
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=0, atol=1e-14)


def test_closed_forms():
    n, c, d, h, w = 1, 4, 2, 2, 2
    lab = RNG.integers(0, c, size=(n, d, h, w))
    loss, dz = orc.softmax_xent_fwd_bwd(Slab(np.full((n, c, d, h, w), 0.7)), lab)
    assert abs(loss - np.log(c)) < 1e-14
    onehot = np.eye(c)[lab].transpose(0, 4, 1, 2, 3)
    np.testing.assert_allclose(dz, (1.0 / c - onehot) / (d * h * w), atol=1e-15)
    z = -50.0 * np.ones((n, c, d, h, w)) + 100.0 * onehot        # the right class wins by a margin of 100
    loss, dz = orc.softmax_xent_fwd_bwd(Slab(z), lab)
    assert 0.0 <= loss < 1e-40 and np.abs(dz).max() < 1e-40


def test_shift_invariance_zero_sum_and_large_logits():
    z, lab = case()
    l0, g0 = orc.softmax_xent_fwd_bwd(Slab(z), lab)
    shift = RNG.normal(0, 300.0, size=(z.shape[0], 1, *z.shape[2:]))          # would overflow exp() without the maximum
    l1, g1 = orc.softmax_xent_fwd_bwd(Slab(z + shift), lab)
    assert abs(l0 - l1) < 1e-11 and np.abs(g0 - g1).max() < 1e-13
    assert np.abs(g0.sum(axis=1)).max() < 1e-16


def test_central_differences():
    z, lab = case(n=1, c=3, d=2, h=2, w=3)
    _, g = orc.softmax_xent_fwd_bwd(Slab(z), lab)
    eps = 1e-6
    for idx in [(0, 0, 0, 0, 0), (0, 2, 1, 1, 2), (0, 1, 0, 1, 1)]:
        zp, zm = z.copy(), z.copy()
        zp[idx] += eps
        zm[idx] -= eps
        fd = (orc.softmax_xent_fwd_bwd(Slab(zp), lab)[0] - orc.softmax_xent_fwd_bwd(Slab(zm), lab)[0]) / (2 * eps)
        assert abs(fd - g[idx]) < 1e-9


def test_shards_add_up_and_halos_are_ignored():
    z, lab = case(n=2, c=3, d=8, h=2, w=4)
    count = lab.size
    full_loss, full_g = orc.softmax_xent_fwd_bwd(Slab(z), lab)
    total = 0.0
    for s in range(4):
        a = np.full((2, 3, 4, 2, 4), np.nan)                      # halo 1/1 holds NaN: must not be touched
        a[:, :, 1:3] = z[:, :, 2 * s:2 * s + 2]
        loss, g = orc.softmax_xent_fwd_bwd(Slab(a, 1, 1, 2 * s, 8), lab[:, 2 * s:2 * s + 2], count)
        total += loss
        np.testing.assert_array_equal(g, full_g[:, :, 2 * s:2 * s + 2])
    assert abs(total - full_loss) < 1e-14


def test_voxels_without_a_class():
    z, lab = case(n=1, c=3, d=2, h=2, w=4)
    count = lab.size
    skip = np.zeros(lab.shape, dtype=bool)
    skip[0, 0, 1, :2] = True
    lab2 = np.where(skip, 255, lab)
    loss, g = orc.softmax_xent_fwd_bwd(Slab(z), lab2, count)
    # the same as masking the per-voxel terms of torch's unreduced loss by hand
    zt = torch.tensor(z, requires_grad=True)
    per = torch.nn.functional.cross_entropy(zt, torch.tensor(lab), reduction="none")
    ref = (per * torch.tensor(~skip)).sum() / count
    ref.backward()
    assert abs(loss - ref.item()) < 1e-13
    np.testing.assert_allclose(g, zt.grad.numpy(), rtol=0, atol=1e-15)
    assert np.all(g[0, :, 0, 1, :2] == 0.0)
