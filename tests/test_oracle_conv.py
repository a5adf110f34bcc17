"""Pins for the CPU oracle's convolution passes (no GPU).

The paper prints no worked numeric example of a layer, so the oracle is pinned
by what mathematics fixes: an independently written brute-force definition, a
library routine (torch CPU float64 + autograd), the impulse identity, closed
forms, linearity, the adjoint identity, finite differences, bit-exact shard
consistency, and the conv-op / parameter totals printed in Table I.
"""
import itertools
import os

import numpy as np
import pytest

import oracle as orc
from oracle import Slab

RNG = np.random.default_rng(12856)


def rand(*shape):
    return RNG.uniform(-1.0, 1.0, size=shape)


# ---------------------------------------------------------------- independent definitions

def brute_fwd(x, w, b):
    """y[n,co,d,h,w] by explicit zero padding and python loops over taps (tiny sizes only)."""
    N, Ci, D, H, W = x.shape
    Co = w.shape[0]
    xp = np.zeros((N, Ci, D + 2, H + 2, W + 2))
    xp[:, :, 1:-1, 1:-1, 1:-1] = x
    y = np.zeros((N, Co, D, H, W))
    for n, co, d, h, v in itertools.product(range(N), range(Co), range(D), range(H), range(W)):
        y[n, co, d, h, v] = b[co] + np.sum(w[co] * xp[n, :, d:d + 3, h:h + 3, v:v + 3])
    return y


def toeplitz_matrix(w, D, H, W):
    """Dense matrix T with vec(y) = T vec(x) for one sample, built tap by tap."""
    Co, Ci = w.shape[:2]
    T = np.zeros((Co * D * H * W, Ci * D * H * W))
    for co, ci, kd, kh, kw in itertools.product(range(Co), range(Ci), range(3), range(3), range(3)):
        for d, h, v in itertools.product(range(D), range(H), range(W)):
            dd, hh, vv = d + kd - 1, h + kh - 1, v + kw - 1
            if 0 <= dd < D and 0 <= hh < H and 0 <= vv < W:
                T[((co * D + d) * H + h) * W + v, ((ci * D + dd) * H + hh) * W + vv] += w[co, ci, kd, kh, kw]
    return T


def leaky(y, a):
    return np.where(y > 0, y, a * y)


# ---------------------------------------------------------------- forward

@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1), (2, 3, 4, 5, 6), (1, 2, 3, 1, 7)])
def test_fwd_brute_force(shape):
    N, Ci, D, H, W = shape
    Co = 3
    x, w, b = rand(*shape), rand(Co, Ci, 3, 3, 3), rand(Co)
    z = orc.conv3d_fwd(Slab(x), w, b)
    np.testing.assert_allclose(z.a, brute_fwd(x, w, b), rtol=0, atol=1e-13)
    z = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.01)
    np.testing.assert_allclose(z.a, leaky(brute_fwd(x, w, b), 0.01), rtol=0, atol=1e-13)
    z = orc.conv3d_fwd(Slab(x), w, None, act=orc.ACT_RELU)
    np.testing.assert_allclose(z.a, np.maximum(brute_fwd(x, w, 0 * b), 0), rtol=0, atol=1e-13)


def test_fwd_toeplitz_and_transpose_is_bwd_data():
    Ci, Co, D, H, W = 2, 3, 3, 4, 5
    x, w, g = rand(1, Ci, D, H, W), rand(Co, Ci, 3, 3, 3), rand(1, Co, D, H, W)
    T = toeplitz_matrix(w, D, H, W)
    z = orc.conv3d_fwd(Slab(x), w, None)
    np.testing.assert_allclose(z.a.ravel(), T @ x.ravel(), atol=1e-13)
    dx = orc.conv3d_bwd_data(Slab(g), None, w)
    np.testing.assert_allclose(dx.a.ravel(), T.T @ g.ravel(), atol=1e-13)


def test_delta_identity_reproduces_flipped_kernel():
    Ci, Co, D, H, W = 3, 2, 5, 6, 7
    w = rand(Co, Ci, 3, 3, 3)
    ci0, p0 = 1, (2, 3, 3)
    x = np.zeros((1, Ci, D, H, W))
    x[0, ci0, p0[0], p0[1], p0[2]] = 1.0
    z = orc.conv3d_fwd(Slab(x), w, None).a
    expect = np.zeros_like(z)
    for kd, kh, kw in itertools.product(range(3), repeat=3):
        expect[0, :, p0[0] + 1 - kd, p0[1] + 1 - kh, p0[2] + 1 - kw] = w[:, ci0, kd, kh, kw]
    assert np.array_equal(z, expect)
    # the 3x3x3 neighbourhood of the impulse, read in array order, is the kernel reversed on every axis
    nb = z[0, :, p0[0] - 1:p0[0] + 2, p0[1] - 1:p0[1] + 2, p0[2] - 1:p0[2] + 2]
    assert np.array_equal(nb, w[:, ci0, ::-1, ::-1, ::-1])
    # impulse in a corner: truncated at the faces
    x[:] = 0
    x[0, 0, 0, 0, 0] = 1.0
    z = orc.conv3d_fwd(Slab(x), w, None).a
    assert np.array_equal(z[0, :, 0:2, 0:2, 0:2], w[:, 0, 1::-1, 1::-1, 1::-1])
    assert np.count_nonzero(z) <= Co * 8


def test_constant_input_closed_form():
    Ci, Co, D, H, W = 4, 2, 4, 5, 6
    z = orc.conv3d_fwd(Slab(np.ones((1, Ci, D, H, W))), np.ones((Co, Ci, 3, 3, 3)), None).a

    def cnt(i, n):
        return 3 - (i == 0) - (i == n - 1)
    for d, h, v in itertools.product(range(D), range(H), range(W)):
        assert z[0, 0, d, h, v] == Ci * cnt(d, D) * cnt(h, H) * cnt(v, W)
    assert z[0, 1, 1, 2, 2] == 27 * Ci and z[0, 0, 0, 2, 2] == 18 * Ci
    assert z[0, 0, 0, 0, 2] == 12 * Ci and z[0, 0, 0, 0, 0] == 8 * Ci


def test_linearity_and_bias():
    x1, x2 = rand(2, 3, 4, 4, 4), rand(2, 3, 4, 4, 4)
    w1, w2, b = rand(5, 3, 3, 3, 3), rand(5, 3, 3, 3, 3), rand(5)
    f = lambda x, w, bb=None: orc.conv3d_fwd(Slab(x), w, bb).a
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, w1), 2 * f(x1, w1) - 3 * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, w1 + 0.5 * w2), f(x1, w1) + 0.5 * f(x1, w2), atol=1e-12)
    np.testing.assert_allclose(f(x1, w1, b), f(x1, w1) + b[None, :, None, None, None], atol=1e-13)


def test_centre_tap_is_channel_gemm():
    x = rand(2, 5, 3, 4, 5)
    A = rand(7, 5)
    w = np.zeros((7, 5, 3, 3, 3))
    w[:, :, 1, 1, 1] = A
    z = orc.conv3d_fwd(Slab(x), w, None).a
    np.testing.assert_allclose(z, np.einsum("oc,ncdhw->nodhw", A, x), atol=1e-13)


def test_separable_kernel_is_three_1d_correlations():
    x = rand(1, 1, 6, 7, 8)
    a, b, c = rand(3), rand(3), rand(3)
    w = np.einsum("i,j,k->ijk", a, b, c)[None, None]
    z = orc.conv3d_fwd(Slab(x), w, None).a[0, 0]

    def corr1d(t, k, axis):
        t = np.moveaxis(t, axis, -1)
        tp = np.pad(t, [(0, 0)] * (t.ndim - 1) + [(1, 1)])
        out = k[0] * tp[..., :-2] + k[1] * tp[..., 1:-1] + k[2] * tp[..., 2:]
        return np.moveaxis(out, -1, axis)
    np.testing.assert_allclose(z, corr1d(corr1d(corr1d(x[0, 0], a, 0), b, 1), c, 2), atol=1e-13)


def test_activation_values():
    # 1x1x1 volume, centre tap 1: z = act(x)
    w = np.zeros((1, 1, 3, 3, 3))
    w[0, 0, 1, 1, 1] = 1.0
    for v, exp in [(-1.0, -0.25), (0.0, 0.0), (1.0, 1.0)]:
        z = orc.conv3d_fwd(Slab(np.full((1, 1, 1, 1, 1), v)), w, None, act=orc.ACT_LEAKY, alpha=0.25).a
        assert z.item() == exp
    assert orc.conv3d_fwd(Slab(np.full((1, 1, 1, 1, 1), -2.0)), w, None, act=orc.ACT_RELU).a.item() == 0.0


# ---------------------------------------------------------------- library cross-check (torch CPU fp64 + autograd)

@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_LEAKY, orc.ACT_RELU])
def test_against_torch_autograd(act):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    N, Ci, Co, D, H, W = 2, 3, 4, 5, 6, 7
    alpha = 0.01
    x, w, b, dz = rand(N, Ci, D, H, W), rand(Co, Ci, 3, 3, 3), rand(Co), rand(N, Co, D, H, W)
    tx, tw, tb = (torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in (x, w, b))
    y = F.conv3d(tx, tw, tb, stride=1, padding=1)
    tz = {orc.ACT_NONE: y, orc.ACT_LEAKY: F.leaky_relu(y, alpha), orc.ACT_RELU: F.relu(y)}[act]
    tz.backward(torch.tensor(dz))
    z = orc.conv3d_fwd(Slab(x), w, b, act=act, alpha=alpha)
    np.testing.assert_allclose(z.a, tz.detach().numpy(), atol=1e-13)
    dx = orc.conv3d_bwd_data(Slab(dz), z, w, act=act, alpha=alpha)
    np.testing.assert_allclose(dx.a, tx.grad.numpy(), atol=1e-12)
    dw, db = orc.conv3d_bwd_filter(Slab(x), Slab(dz), z, act=act, alpha=alpha)
    np.testing.assert_allclose(dw, tw.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), atol=1e-11)


# ---------------------------------------------------------------- backward passes

def test_adjoint_identity_unsharded_and_slab():
    Ci, Co, D, H, W = 3, 4, 8, 5, 6
    w = rand(Co, Ci, 3, 3, 3)
    x, g = rand(2, Ci, D, H, W), rand(2, Co, D, H, W)
    lhs = np.sum(orc.conv3d_fwd(Slab(x), w, None).a * g)
    rhs = np.sum(x * orc.conv3d_bwd_data(Slab(g), None, w).a)
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)
    # slab form: <conv(x), g> summed over shards equals <x, bwd_data(g)> summed over shards
    lhs_s = rhs_s = 0.0
    for off in (0, 4):
        xs = cut(x, off, 4, 1)
        gs = cut(g, off, 4, 1)
        lhs_s += np.sum(orc.conv3d_fwd(xs, w, None).interior * gs.interior)
        rhs_s += np.sum(xs.interior * orc.conv3d_bwd_data(gs, None, w).interior)
    assert abs(lhs_s - lhs) <= 1e-12 * abs(lhs) and abs(rhs_s - lhs) <= 1e-12 * abs(lhs)


def test_bwd_filter_finite_differences_and_impulse():
    Ci, Co, D, H, W = 2, 3, 4, 4, 5
    x, w, g = rand(1, Ci, D, H, W), rand(Co, Ci, 3, 3, 3), rand(1, Co, D, H, W)
    dw, db = orc.conv3d_bwd_filter(Slab(x), Slab(g), None)
    L = lambda ww, bb: np.sum(orc.conv3d_fwd(Slab(x), ww, bb).a * g)
    b0 = rand(Co)
    eps = 0.5  # L is linear in w and b: central differences are exact up to rounding
    for idx in [(0, 0, 0, 0, 0), (2, 1, 1, 1, 1), (1, 0, 2, 0, 1), (0, 1, 0, 2, 2), (2, 1, 2, 2, 2)]:
        e = np.zeros_like(w)
        e[idx] = eps
        fd = (L(w + e, b0) - L(w - e, b0)) / (2 * eps)
        assert abs(fd - dw[idx]) <= 1e-11 * max(1.0, abs(fd))
    for co in range(Co):
        e = np.zeros(Co)
        e[co] = eps
        fd = (L(w, b0 + e) - L(w, b0 - e)) / (2 * eps)
        assert abs(fd - db[co]) <= 1e-11 * max(1.0, abs(fd))
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3, 4)), atol=1e-12)
    # g = impulse at (co0, p0)  =>  dw[co0, ci, k] = x~[ci, p0 + k - 1]: reads the input patch back
    g0 = np.zeros_like(g)
    co0, p0 = 1, (0, 2, 4)
    g0[0, co0, p0[0], p0[1], p0[2]] = 1.0
    dw0, _ = orc.conv3d_bwd_filter(Slab(x), Slab(g0), None)
    xp = np.pad(x, [(0, 0), (0, 0), (1, 1), (1, 1), (1, 1)])
    assert np.array_equal(dw0[co0], xp[0, :, p0[0]:p0[0] + 3, p0[1]:p0[1] + 3, p0[2]:p0[2] + 3])
    assert not dw0[[0, 2]].any()


def test_masked_backward_uses_saved_output_sign():
    Ci, Co = 2, 2
    x, w, b, dz = rand(1, Ci, 3, 4, 4), rand(Co, Ci, 3, 3, 3), rand(Co), rand(1, Co, 3, 4, 4)
    z = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.1)
    g = dz * np.where(z.a > 0, 1.0, 0.1)
    a = orc.conv3d_bwd_data(Slab(dz), z, w, act=orc.ACT_LEAKY, alpha=0.1).a
    bq = orc.conv3d_bwd_data(Slab(g), None, w).a
    assert np.array_equal(a, bq)
    dwa, dba = orc.conv3d_bwd_filter(Slab(x), Slab(dz), z, act=orc.ACT_LEAKY, alpha=0.1)
    dwb, dbb = orc.conv3d_bwd_filter(Slab(x), Slab(g), None)
    assert np.array_equal(dwa, dwb) and np.array_equal(dba, dbb)


# ---------------------------------------------------------------- slab form

def cut(full, off, d, halo, halo_out_of_volume_fill=0.0):
    """Slab [off, off+d) of `full` with `halo` stored planes per side (outside the volume: a canary, never read)."""
    N, C, Dg, H, W = full.shape
    a = np.full((N, C, d + 2 * halo, H, W), halo_out_of_volume_fill)
    for i, g in enumerate(range(off - halo, off + d + halo)):
        if 0 <= g < Dg:
            a[:, :, i] = full[:, :, g]
    return Slab(a, halo, halo, off, Dg)


@pytest.mark.parametrize("nshard", [1, 2, 4])
def test_shard_consistency_bit_exact(nshard):
    Ci, Co, Dg, H, W = 3, 4, 8, 5, 6
    x, w, b, dz = rand(2, Ci, Dg, H, W), rand(Co, Ci, 3, 3, 3), rand(Co), rand(2, Co, Dg, H, W)
    zf = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.01)
    dxf = orc.conv3d_bwd_data(Slab(dz), zf, w, act=orc.ACT_LEAKY, alpha=0.01)
    dwf, dbf = orc.conv3d_bwd_filter(Slab(x), Slab(dz), zf, act=orc.ACT_LEAKY, alpha=0.01)
    d = Dg // nshard
    dws, dbs = 0.0, 0.0
    for s in range(nshard):
        off = s * d
        # halo planes outside the global volume hold NaN: the oracle must never read them
        xs = cut(x, off, d, 1, np.nan)
        zs = orc.conv3d_fwd(xs, w, b, act=orc.ACT_LEAKY, alpha=0.01)
        assert np.array_equal(zs.a, zf.a[:, :, off:off + d])
        dzs, zs1 = cut(dz, off, d, 1, np.nan), cut(zf.a, off, d, 1, np.nan)
        dxs = orc.conv3d_bwd_data(dzs, zs1, w, act=orc.ACT_LEAKY, alpha=0.01)
        assert np.array_equal(dxs.a, dxf.a[:, :, off:off + d])
        dw, db = orc.conv3d_bwd_filter(xs, cut(dz, off, d, 0), cut(zf.a, off, d, 0), act=orc.ACT_LEAKY, alpha=0.01)
        dws, dbs = dws + dw, dbs + db
    np.testing.assert_allclose(dws, dwf, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dbs, dbf, rtol=1e-12, atol=1e-12)


def test_halo_recompute_and_out_of_volume_planes_are_zero():
    """A 2-plane halo serves two stacked convs: conv-a also produces the first halo plane of its output."""
    Ci, Cm, Co, Dg, H, W = 1, 3, 2, 8, 4, 5
    x, wa, ba, wb = rand(1, Ci, Dg, H, W), rand(Cm, Ci, 3, 3, 3), rand(Cm), rand(Co, Cm, 3, 3, 3)
    ya = orc.conv3d_fwd(Slab(x), wa, ba, act=orc.ACT_RELU)
    yb = orc.conv3d_fwd(ya, wb, None)
    for off in (0, 4):
        xs = cut(x, off, 4, 2, np.nan)
        a = orc.conv3d_fwd(xs, wa, ba, cout_halo=(1, 1), act=orc.ACT_RELU)
        # the plane beyond the global boundary is the next layer's zero padding, not act(bias)
        if off == 0:
            assert not a.a[:, :, 0].any()
        else:
            assert not a.a[:, :, -1].any()
        bq = orc.conv3d_fwd(a, wb, None)
        assert np.array_equal(bq.a, yb.a[:, :, off:off + 4])


def test_missing_halo_is_an_error():
    x = cut(rand(1, 1, 8, 3, 3), 4, 2, 0)
    with pytest.raises(ValueError):
        orc.conv3d_fwd(x, rand(1, 1, 3, 3, 3), None)


# ---------------------------------------------------------------- Table I bookkeeping

def test_table1_conv_ops_and_parameters():
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_network.txt")
    conv, fc, printed = [], [], {}
    for line in open(path):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "conv":
            conv.append((int(t[2]), int(t[3]), [int(v) for v in t[4:7]]))
        elif t[0] == "fc":
            fc.append((int(t[2]), int(t[3])))
        elif t[0] == "printed":
            printed[t[1]] = [float(v) for v in t[2:5]]
    for col in range(3):
        fwd = sum(orc.conv_flops(ci, co, wd[col] ** 3) for ci, co, wd in conv)
        # the table prints 4 significant digits
        assert f"{fwd / 1e9:.4g}" == f"{printed['fwd_gflop'][col]:.4g}"
        assert f"{3 * fwd / 1e9:.4g}" == f"{printed['total_gflop'][col]:.4g}"
    params = sum(27 * ci * co for ci, co, _ in conv) + sum(i * o + o for i, o in fc)
    assert f"{params / 1e6:.2f}" == f"{printed['params_1e6'][0]:.2f}"


def test_act_bwd_equals_the_fused_mask():
    """The separate activation-backward pass followed by an unmasked BD/BF equals the fused form."""
    x, w, b = rand(1, 2, 4, 4, 5), rand(3, 2, 3, 3, 3), rand(3)
    dz, dz2 = rand(1, 3, 4, 4, 5), rand(1, 3, 4, 4, 5)
    z = orc.conv3d_fwd(Slab(x), w, b, act=orc.ACT_LEAKY, alpha=0.2)
    g = orc.act_bwd(Slab(dz), None, z, orc.ACT_LEAKY, 0.2)
    assert np.array_equal(orc.conv3d_bwd_data(g, None, w).a, orc.conv3d_bwd_data(Slab(dz), z, w, act=orc.ACT_LEAKY, alpha=0.2).a)
    dw_a, db_a = orc.conv3d_bwd_filter(Slab(x), g, None)
    dw_b, db_b = orc.conv3d_bwd_filter(Slab(x), Slab(dz), z, act=orc.ACT_LEAKY, alpha=0.2)
    assert np.array_equal(dw_a, dw_b) and np.array_equal(db_a, db_b)
    g2 = orc.act_bwd(Slab(dz), Slab(dz2), z, orc.ACT_RELU)
    assert np.array_equal(g2.a, (dz + dz2) * (z.a > 0))
    assert np.array_equal(orc.act_bwd(Slab(dz), None, z, orc.ACT_NONE).a, dz)
