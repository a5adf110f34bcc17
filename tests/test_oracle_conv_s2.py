"""Pins for the oracle's stride-2 convolution (Table I, fourth convolution), no GPU.

What fixes it: (i) with one zero voxel of padding on every side the stride-2 output is the stride-1
output sampled at the even positions (the stride-1 oracle is pinned on its own); (ii) a library routine
(torch CPU float64, stride 2, padding 1, with autograd for both gradients); (iii) the adjoint identity
between forward and backward-data; (iv) a brute-force loop over padded windows; (v) the delta input;
(vi) bit-exact shard consistency, with the halo sides the two directions need.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle as orc
from oracle import Slab

RNG = np.random.default_rng(2007_12856 + 2)


def rand(*shape):
    return RNG.uniform(-1.0, 1.0, size=shape)


SHAPES = [(1, 1, 2, 2, 2), (2, 3, 4, 6, 8), (1, 2, 6, 5, 7), (1, 4, 2, 1, 3)]


@pytest.mark.parametrize("shape", SHAPES)
def test_fwd_is_stride1_at_even_positions(shape):
    N, Ci, D, H, W = shape
    x, w, b = rand(*shape), rand(3, Ci, 3, 3, 3), rand(3)
    y2 = orc.conv3d_s2_fwd(Slab(x), w, b, orc.ACT_LEAKY, 0.1).a
    y1 = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.1).a
    assert y2.shape == (N, 3, D // 2, (H + 1) // 2, (W + 1) // 2)
    np.testing.assert_allclose(y2, y1[:, :, ::2, ::2, ::2], rtol=0, atol=1e-13)


def test_fwd_brute_force_windows():
    N, Ci, D, H, W, Co = 1, 2, 4, 3, 6, 2
    x, w, b = rand(N, Ci, D, H, W), rand(Co, Ci, 3, 3, 3), rand(Co)
    xp = np.zeros((N, Ci, D + 2, H + 2, W + 2))
    xp[:, :, 1:-1, 1:-1, 1:-1] = x
    y = orc.conv3d_s2_fwd(Slab(x), w, b).a
    for co, d, h, v in itertools.product(range(Co), range(D // 2), range((H + 1) // 2), range(W // 2)):
        ref = b[co] + np.sum(w[co] * xp[0, :, 2 * d:2 * d + 3, 2 * h:2 * h + 3, 2 * v:2 * v + 3])
        assert abs(y[0, co, d, h, v] - ref) < 1e-13


def test_delta_input_reads_the_filter_back():
    # x = delta at an odd position (3,3,3): output voxel p sees it through tap k = 3 - 2p + 1, p in {1, 2}
    Ci, Co = 2, 3
    x = np.zeros((1, Ci, 8, 8, 8))
    x[0, 1, 3, 3, 3] = 1.0
    w = rand(Co, Ci, 3, 3, 3)
    y = orc.conv3d_s2_fwd(Slab(x), w, None).a
    ref = np.zeros_like(y)
    for pd, ph, pw in itertools.product((1, 2), repeat=3):
        ref[0, :, pd, ph, pw] = w[:, 1, 4 - 2 * pd, 4 - 2 * ph, 4 - 2 * pw]
    np.testing.assert_array_equal(y, ref)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_LEAKY])
def test_all_three_passes_match_torch_float64(shape, act):
    N, Ci, D, H, W = shape
    Co = 3
    x, w, b = rand(*shape), rand(Co, Ci, 3, 3, 3), rand(Co)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    yt = torch.nn.functional.conv3d(xt, wt, bt, stride=2, padding=1)
    if act == orc.ACT_LEAKY:
        yt = torch.nn.functional.leaky_relu(yt, 0.1)
    y = orc.conv3d_s2_fwd(Slab(x), w, b, act, 0.1)
    np.testing.assert_allclose(y.a, yt.detach().numpy(), rtol=0, atol=1e-12)
    dy = rand(*y.a.shape)
    yt.backward(torch.tensor(dy))
    dx = orc.conv3d_s2_bwd_data(Slab(dy), y, w, Slab(x), act, 0.1)
    np.testing.assert_allclose(dx.a, xt.grad.numpy(), rtol=0, atol=1e-12)
    dw, db = orc.conv3d_s2_bwd_filter(Slab(x), Slab(dy), y, act, 0.1)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=0, atol=1e-12)


def test_adjoint_identity():
    x, w = rand(2, 3, 6, 4, 8), rand(4, 3, 3, 3, 3)
    y = orc.conv3d_s2_fwd(Slab(x), w, None)
    g = rand(*y.a.shape)
    dx = orc.conv3d_s2_bwd_data(Slab(g), None, w, Slab(x))
    lhs, rhs = np.sum(y.a * g), np.sum(x * dx.a)
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def _cut(full, lo, hi, halo_lo, halo_hi, d_global):
    """Slab [lo,hi) of a full tensor with the given halo widths; planes outside the volume hold a canary."""
    N, C, D, H, W = full.shape
    a = np.full((N, C, halo_lo + hi - lo + halo_hi, H, W), 777.0)
    for s in range(a.shape[2]):
        gp = lo - halo_lo + s
        if 0 <= gp < D:
            a[:, :, s] = full[:, :, gp]
    return Slab(a, halo_lo, halo_hi, lo, d_global)


@pytest.mark.parametrize("shards", [2, 4])
def test_shards_reproduce_the_unsharded_result(shards):
    N, Ci, Co, D, H, W = 1, 2, 3, 16, 4, 6
    x, w, b = rand(N, Ci, D, H, W), rand(Co, Ci, 3, 3, 3), rand(Co)
    full_y = orc.conv3d_s2_fwd(Slab(x), w, b, orc.ACT_LEAKY, 0.2)
    dy = rand(*full_y.a.shape)
    full_dx = orc.conv3d_s2_bwd_data(Slab(dy), full_y, w, Slab(x), orc.ACT_LEAKY, 0.2)
    full_dw, full_db = orc.conv3d_s2_bwd_filter(Slab(x), Slab(dy), full_y, orc.ACT_LEAKY, 0.2)
    d = D // shards
    dw_sum, db_sum = 0.0, 0.0
    for s in range(shards):
        xs = _cut(x, s * d, (s + 1) * d, 1, 0, D)                     # forward / filter: lower halo only
        ys = orc.conv3d_s2_fwd(xs, w, b, orc.ACT_LEAKY, 0.2)
        np.testing.assert_array_equal(ys.a, full_y.a[:, :, s * d // 2:(s + 1) * d // 2])
        dys = _cut(dy, s * d // 2, (s + 1) * d // 2, 0, 1, D // 2)    # backward-data: upper halo only
        yss = _cut(full_y.a, s * d // 2, (s + 1) * d // 2, 0, 1, D // 2)
        dxs = orc.conv3d_s2_bwd_data(dys, yss, w, Slab(xs.interior, 0, 0, s * d, D), orc.ACT_LEAKY, 0.2)
        np.testing.assert_array_equal(dxs.a, full_dx.a[:, :, s * d:(s + 1) * d])
        dw, db = orc.conv3d_s2_bwd_filter(xs, dys, yss, orc.ACT_LEAKY, 0.2)
        dw_sum, db_sum = dw_sum + dw, db_sum + db
    np.testing.assert_allclose(dw_sum, full_dw, rtol=0, atol=1e-12)
    np.testing.assert_allclose(db_sum, full_db, rtol=0, atol=1e-12)


def test_missing_halo_is_an_error():
    x, w = rand(1, 1, 4, 4, 4), rand(1, 1, 3, 3, 3)
    with pytest.raises(ValueError):
        orc.conv3d_s2_fwd(Slab(x, 0, 0, 4, 8), w, None)               # interior shard without its lower halo
    y = orc.conv3d_s2_fwd(Slab(x), w, None)
    with pytest.raises(ValueError):
        orc.conv3d_s2_bwd_data(Slab(y.a, 0, 0, 0, 4), None, w, Slab(x, 0, 0, 0, 8))   # lower shard without dy's upper halo
