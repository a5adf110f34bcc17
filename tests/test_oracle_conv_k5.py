"""Pins for the oracle's 5x5x5 convolution (Sec. III-A: 3^3 and 5^3 filters; halo of two planes), no GPU.

What fixes it: (i) the odd-edge functions at K = 3 give the 3x3x3 oracle (pinned on its own); (ii) a 3x3x3
filter embedded in the middle of a zero 5x5x5 filter gives the 3x3x3 result; (iii) a library routine (torch
CPU float64, padding 2, with autograd for both gradients); (iv) a brute-force loop over padded windows;
(v) the delta input reads the reversed filter back; (vi) the adjoint identity between forward and
backward-data; (vii) shard consistency with two halo planes per side, partial filter gradients adding up.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle as orc
from oracle import Slab

RNG = np.random.default_rng(2007_12856 + 5)


def rand(*shape):
    return RNG.uniform(-1.0, 1.0, size=shape)


SHAPES = [(1, 1, 1, 1, 1), (2, 3, 4, 6, 8), (1, 2, 7, 5, 3), (1, 4, 2, 9, 6)]


@pytest.mark.parametrize("shape", SHAPES)
def test_k3_is_the_3x3x3_oracle(shape):
    N, Ci, D, H, W = shape
    x, w, b, dz = rand(*shape), rand(3, Ci, 3, 3, 3), rand(3), rand(N, 3, D, H, W)
    z3 = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.1)
    zk = orc.convk_fwd(Slab(x), w, b, orc.ACT_LEAKY, 0.1)
    np.testing.assert_array_equal(zk.a, z3.a)
    np.testing.assert_array_equal(orc.convk_bwd_data(Slab(dz), zk, w, orc.ACT_LEAKY, 0.1).a,
                                  orc.conv3d_bwd_data(Slab(dz), z3, w, act=orc.ACT_LEAKY, alpha=0.1).a)
    dwk, dbk = orc.convk_bwd_filter(3, Slab(x), Slab(dz), zk, orc.ACT_LEAKY, 0.1)
    dw3, db3 = orc.conv3d_bwd_filter(Slab(x), Slab(dz), z3, orc.ACT_LEAKY, 0.1)
    np.testing.assert_array_equal(dwk, dw3)
    np.testing.assert_array_equal(dbk, db3)


@pytest.mark.parametrize("shape", SHAPES[1:])
def test_embedded_3x3x3_filter(shape):
    N, Ci, D, H, W = shape
    x, w3, b, dz = rand(*shape), rand(2, Ci, 3, 3, 3), rand(2), rand(N, 2, D, H, W)
    w5 = np.zeros((2, Ci, 5, 5, 5))
    w5[:, :, 1:4, 1:4, 1:4] = w3
    np.testing.assert_allclose(orc.convk_fwd(Slab(x), w5, b).a, orc.conv3d_fwd(Slab(x), w3, b).a, rtol=0, atol=1e-13)
    np.testing.assert_allclose(orc.convk_bwd_data(Slab(dz), None, w5).a, orc.conv3d_bwd_data(Slab(dz), None, w3).a,
                               rtol=0, atol=1e-13)
    dw5, db5 = orc.convk_bwd_filter(5, Slab(x), Slab(dz), None)
    dw3, db3 = orc.conv3d_bwd_filter(Slab(x), Slab(dz), None)
    np.testing.assert_allclose(dw5[:, :, 1:4, 1:4, 1:4], dw3, rtol=0, atol=1e-12)
    np.testing.assert_allclose(db5, db3, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("act,alpha", [(orc.ACT_NONE, 0.0), (orc.ACT_RELU, 0.0), (orc.ACT_LEAKY, 0.25)])
def test_against_torch_float64_with_autograd(shape, act, alpha):
    N, Ci, D, H, W = shape
    Co = 3
    x, w, b, dz = rand(*shape), rand(Co, Ci, 5, 5, 5), rand(Co), rand(N, Co, D, H, W)
    xt, wt, bt = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, w, b))
    y = torch.nn.functional.conv3d(xt, wt, bt, stride=1, padding=2)
    if act == orc.ACT_RELU:
        y = torch.relu(y)
    elif act == orc.ACT_LEAKY:
        y = torch.nn.functional.leaky_relu(y, alpha)
    y.backward(torch.tensor(dz))
    z = orc.convk_fwd(Slab(x), w, b, act, alpha)
    np.testing.assert_allclose(z.a, y.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(orc.convk_bwd_data(Slab(dz), z, w, act, alpha).a, xt.grad.numpy(), rtol=0, atol=1e-12)
    dw, db = orc.convk_bwd_filter(5, Slab(x), Slab(dz), z, act, alpha)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=0, atol=1e-11)


def test_fwd_brute_force_windows():
    N, Ci, D, H, W, Co = 1, 2, 3, 4, 6, 2
    x, w, b = rand(N, Ci, D, H, W), rand(Co, Ci, 5, 5, 5), rand(Co)
    xp = np.zeros((N, Ci, D + 4, H + 4, W + 4))
    xp[:, :, 2:-2, 2:-2, 2:-2] = x
    z = orc.convk_fwd(Slab(x), w, b).a
    for co, d, h, v in itertools.product(range(Co), range(D), range(H), range(W)):
        ref = b[co] + np.sum(w[co] * xp[0, :, d:d + 5, h:h + 5, v:v + 5])
        assert abs(z[0, co, d, h, v] - ref) < 1e-13


def test_delta_input_reads_the_reversed_filter_back():
    Ci, Co = 2, 3
    x = np.zeros((1, Ci, 7, 8, 9))
    x[0, 1, 3, 4, 5] = 1.0
    w = rand(Co, Ci, 5, 5, 5)
    z = orc.convk_fwd(Slab(x), w, None).a
    ref = np.zeros_like(z)
    # output voxel p sees the delta through tap k = c - p + 2
    ref[0, :, 1:6, 2:7, 3:8] = w[:, 1, ::-1, ::-1, ::-1]
    np.testing.assert_array_equal(z, ref)


def test_adjoint_identity():
    shape = (2, 3, 5, 6, 7)
    x, w, dz = rand(*shape), rand(4, 3, 5, 5, 5), rand(2, 4, 5, 6, 7)
    lhs = np.sum(orc.convk_fwd(Slab(x), w, None).a * dz)
    rhs = np.sum(x * orc.convk_bwd_data(Slab(dz), None, w).a)
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


def _shards(a, cuts, halo):
    D = a.shape[2]
    out = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        hl, hh = min(halo, lo), min(halo, D - hi)
        out.append(Slab(a[:, :, lo - hl:hi + hh].copy(), hl, hh, lo, D))
    return out


def test_shards_with_two_halo_planes_reproduce_the_whole_volume():
    N, Ci, Co, D, H, W = 2, 2, 3, 9, 5, 6
    x, w, b, dz = rand(N, Ci, D, H, W), rand(Co, Ci, 5, 5, 5), rand(Co), rand(N, Co, D, H, W)
    act, alpha = orc.ACT_LEAKY, 0.1
    z = orc.convk_fwd(Slab(x), w, b, act, alpha)
    dx = orc.convk_bwd_data(Slab(dz), z, w, act, alpha)
    dw, db = orc.convk_bwd_filter(5, Slab(x), Slab(dz), z, act, alpha)
    cuts = [0, 2, 5, 9]          # a 2-plane shard: its neighbours' neighbours are not needed with a halo of 2
    dw_sum, db_sum = np.zeros_like(dw), np.zeros_like(db)
    for xs, dzs, zs, dzi, zi in zip(_shards(x, cuts, 2), _shards(dz, cuts, 2), _shards(z.a, cuts, 2),
                                    _shards(dz, cuts, 0), _shards(z.a, cuts, 0)):
        lo = xs.d_offset
        np.testing.assert_array_equal(orc.convk_fwd(xs, w, b, act, alpha).a, z.a[:, :, lo:lo + xs.d])
        np.testing.assert_array_equal(orc.convk_bwd_data(dzs, zs, w, act, alpha).a, dx.a[:, :, lo:lo + xs.d])
        pdw, pdb = orc.convk_bwd_filter(5, xs, dzi, zi, act, alpha)
        dw_sum += pdw
        db_sum += pdb
    np.testing.assert_allclose(dw_sum, dw, rtol=0, atol=1e-12)
    np.testing.assert_allclose(db_sum, db, rtol=0, atol=1e-12)


def test_missing_halo_planes_are_an_error():
    x = Slab(rand(1, 1, 4 + 1 + 2, 3, 3), 1, 2, 4, 16)      # lower halo of one plane only
    with pytest.raises(ValueError):
        orc.convk_fwd(x, rand(1, 1, 5, 5, 5), None)
