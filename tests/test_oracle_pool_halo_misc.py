"""Pins for the oracle's pooling, halo pack/unpack, 2x2x2 transposed conv, concat, dense and loss (no GPU)."""
import itertools

import numpy as np
import pytest

import oracle as orc
from oracle import Slab

RNG = np.random.default_rng(2007)


def rand(*shape):
    return RNG.uniform(-1.0, 1.0, size=shape)


# ---------------------------------------------------------------- pooling

@pytest.mark.parametrize("mode", [orc.POOL_AVG, orc.POOL_MAX])
def test_pool_constant_and_sums(mode):
    x = Slab(np.full((2, 3, 4, 6, 8), 0.75))
    y = orc.pool3d_fwd(x, mode)
    assert y.a.shape == (2, 3, 2, 3, 4) and np.all(y.a == 0.75)
    dy = Slab(rand(2, 3, 2, 3, 4))
    xr = Slab(rand(2, 3, 4, 6, 8))
    dx = orc.pool3d_bwd(dy, xr, mode)
    assert abs(dx.a.sum() - dy.a.sum()) < 1e-12
    # per-window sums are preserved too
    win = dx.a.reshape(2, 3, 2, 2, 3, 2, 4, 2).sum(axis=(3, 5, 7))
    np.testing.assert_allclose(win, dy.a, atol=1e-15)


def test_pool_definition_by_reshape():
    x = rand(1, 2, 4, 4, 6)
    blocks = x.reshape(1, 2, 2, 2, 2, 2, 3, 2)
    assert np.allclose(orc.pool3d_fwd(Slab(x), orc.POOL_AVG).a, blocks.mean(axis=(3, 5, 7)), atol=1e-15)
    assert np.array_equal(orc.pool3d_fwd(Slab(x), orc.POOL_MAX).a, blocks.max(axis=(3, 5, 7)))


def test_avg_pool_adjoint():
    x, g = rand(1, 2, 4, 4, 4), rand(1, 2, 2, 2, 2)
    lhs = np.sum(orc.pool3d_fwd(Slab(x), orc.POOL_AVG).a * g)
    rhs = np.sum(x * orc.pool3d_bwd(Slab(g), None, orc.POOL_AVG).a)
    assert abs(lhs - rhs) < 1e-13


def test_max_pool_tie_goes_to_first_in_row_major_order():
    x = np.zeros((1, 1, 2, 2, 4))
    x[0, 0, :, :, 2:] = [[[1.0, 5.0], [5.0, 2.0]], [[5.0, 0.0], [0.0, 5.0]]]
    dy = np.array([3.0, 7.0]).reshape(1, 1, 1, 1, 2)
    dx = orc.pool3d_bwd(Slab(dy), Slab(x), orc.POOL_MAX).a
    expect = np.zeros_like(x)
    expect[0, 0, 0, 0, 0] = 3.0      # all-equal window: k = (0,0,0)
    expect[0, 0, 0, 0, 3] = 7.0      # first of the four 5.0 in (kd,kh,kw) order is (0,0,1)
    assert np.array_equal(dx, expect)


def test_pool_against_torch():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    x = rand(2, 3, 4, 6, 8)
    g = rand(2, 3, 2, 3, 4)
    for mode, fn in [(orc.POOL_AVG, F.avg_pool3d), (orc.POOL_MAX, F.max_pool3d)]:
        tx = torch.tensor(x, requires_grad=True)
        ty = fn(tx, 2, 2)
        ty.backward(torch.tensor(g))
        np.testing.assert_allclose(orc.pool3d_fwd(Slab(x), mode).a, ty.detach().numpy(), atol=1e-15)
        np.testing.assert_allclose(orc.pool3d_bwd(Slab(g), Slab(x), mode).a, tx.grad.numpy(), atol=1e-15)


def test_pool_on_slab_touches_interior_only_and_matches_full():
    full = rand(1, 2, 8, 4, 4)
    yf = orc.pool3d_fwd(Slab(full), orc.POOL_MAX)
    a = np.full((1, 2, 6, 4, 4), np.nan)
    a[:, :, 1:5] = full[:, :, 4:8]
    ys = orc.pool3d_fwd(Slab(a, 1, 1, 4, 8), orc.POOL_MAX, y_halo=(1, 1))
    assert (ys.d_offset, ys.d_global) == (2, 4)
    assert np.array_equal(ys.interior, yf.a[:, :, 2:4])
    assert not ys.a[:, :, 0].any() and not ys.a[:, :, -1].any()
    with pytest.raises(ValueError):
        orc.pool3d_fwd(Slab(a[:, :, 1:4], 0, 0, 4, 8), orc.POOL_AVG)    # odd depth: window would straddle a face


# ---------------------------------------------------------------- halo pack / unpack

def test_halo_exchange_between_neighbouring_shards_reproduces_full_volume():
    full = rand(2, 3, 12, 4, 5)
    shards = []
    for s in range(3):
        a = np.full((2, 3, 4 + 4, 4, 5), 777.0)     # canary everywhere but the interior
        a[:, :, 2:6] = full[:, :, 4 * s:4 * s + 4]
        shards.append(Slab(a, 2, 2, 4 * s, 12))
    for width in (1, 2):
        for s in range(3):
            lo_buf = orc.halo_pack(shards[s - 1], orc.FACE_D_HI, width) if s > 0 else None
            hi_buf = orc.halo_pack(shards[s + 1], orc.FACE_D_LO, width) if s < 2 else None
            orc.halo_unpack(lo_buf, shards[s], orc.FACE_D_LO, width)
            orc.halo_unpack(hi_buf, shards[s], orc.FACE_D_HI, width)
        for s in range(3):
            t = shards[s]
            for i, g in enumerate(range(4 * s - 2, 4 * s + 6)):
                plane = t.a[:, :, i]
                dist = (4 * s - g) if g < 4 * s else (g - (4 * s + 3) if g > 4 * s + 3 else 0)
                if dist > width:
                    assert np.all(plane == 777.0)           # not addressed: untouched
                elif 0 <= g < 12:
                    assert np.array_equal(plane, full[:, :, g])
                else:
                    assert not plane.any()                   # global boundary: zero fill


def test_pack_layout_and_roundtrip():
    t = Slab(np.arange(2 * 2 * 5 * 2 * 3, dtype=np.float64).reshape(2, 2, 5, 2, 3), 1, 1)
    lo, hi = orc.halo_pack(t, orc.FACE_D_LO, 1), orc.halo_pack(t, orc.FACE_D_HI, 1)
    assert lo.shape == (2, 2, 1, 2, 3)
    assert np.array_equal(lo[:, :, 0], t.a[:, :, 1]) and np.array_equal(hi[:, :, 0], t.a[:, :, 3])
    u = Slab(np.zeros_like(t.a), 1, 1)
    orc.halo_unpack(lo, u, orc.FACE_D_HI, 1)
    assert np.array_equal(orc.halo_pack(Slab(u.a[:, :, 2:], 0, 0), orc.FACE_D_HI, 1), lo)


def test_general_faces_of_a_2x2x2_partition_reproduce_the_full_volume():
    """Sec. II-B partitions the domain in any spatial dimension.  A 2x2x2 grid of sub-domains with a one-voxel halo
    on every side: after every sub-domain has packed its six faces (as wide as the neighbour's halo box needs them,
    in D, then H including the fresh D halos, then W including both: the usual three-phase exchange that also
    fills edges and corners) and the neighbours have unpacked them, each padded block equals the zero-padded full
    volume cut at its place; what no box addresses keeps its canary."""
    N, C, S = 2, 2, 4                     # sub-domain edge
    full = rand(N, C, 2 * S, 2 * S, 2 * S)
    padded = np.zeros((N, C, 2 * S + 2, 2 * S + 2, 2 * S + 2))
    padded[:, :, 1:-1, 1:-1, 1:-1] = full
    blocks = {}
    for bd in range(2):
        for bh in range(2):
            for bw in range(2):
                a = np.full((N, C, S + 2, S + 2, S + 2), 777.0)
                a[:, :, 1:-1, 1:-1, 1:-1] = full[:, :, bd * S:(bd + 1) * S, bh * S:(bh + 1) * S, bw * S:(bw + 1) * S]
                blocks[bd, bh, bw] = a
    E = S + 2
    for axis in range(3):                 # phase 0: D faces of the interior; 1: H faces over the filled D extent; 2: W faces
        for key, a in blocks.items():
            for side in (0, 1):
                nb = list(key)
                nb[axis] += 1 if side else -1
                # the halo box on `side` of this block, and the neighbour's matching interior slice
                lo = [1, 1, 1]; ext = [S, S, S]
                for prev in range(axis):
                    lo[prev], ext[prev] = 0, E
                dst = list(lo); dst_ext = list(ext)
                dst[axis] = E - 1 if side else 0
                dst_ext[axis] = 1
                src = list(lo)
                src[axis] = 1 if side else S
                box_dst = (dst[0], dst[1], dst[2], dst_ext[0], dst_ext[1], dst_ext[2])
                if 0 <= nb[axis] < 2:
                    box_src = (src[0], src[1], src[2], dst_ext[0], dst_ext[1], dst_ext[2])
                    orc.box_unpack(orc.box_pack(blocks[tuple(nb)], box_src), a, box_dst)
                else:
                    orc.box_unpack(None, a, box_dst)
    for (bd, bh, bw), a in blocks.items():
        want = padded[:, :, bd * S:bd * S + E, bh * S:bh * S + E, bw * S:bw * S + E]
        assert np.array_equal(a, want)


def test_box_pack_layout_roundtrip_and_untouched_rest():
    a = np.arange(2 * 3 * 4 * 5 * 6, dtype=np.float64).reshape(2, 3, 4, 5, 6)
    box = (1, 2, 3, 2, 3, 2)
    b = orc.box_pack(a, box)
    assert b.shape == (2, 3, 2, 3, 2)
    assert np.array_equal(b, a[:, :, 1:3, 2:5, 3:5])                   # the library slicing of the same box
    assert b[1, 2, 1, 2, 1] == a[1, 2, 2, 4, 4]
    u = np.full_like(a, -1.0)
    orc.box_unpack(b, u, box)
    assert np.array_equal(orc.box_pack(u, box), b)
    mask = np.ones(a.shape, dtype=bool)
    mask[:, :, 1:3, 2:5, 3:5] = False
    assert np.all(u[mask] == -1.0)
    orc.box_unpack(None, u, (0, 0, 0, 4, 5, 1))                        # a W face on the global boundary
    assert not u[..., 0].any() and np.all(u[..., 1][mask[..., 1]] == -1.0)


# ---------------------------------------------------------------- 2x2x2 stride-2 transposed convolution

def test_deconv_is_adjoint_of_stride2_correlation_and_closed_form():
    Ci, Co = 3, 2
    x, w, y = rand(1, Ci, 2, 3, 2), rand(Ci, Co, 2, 2, 2), rand(1, Co, 4, 6, 4)
    up = orc.deconv2_fwd(Slab(x), w, None)
    # stride-2 correlation written out independently
    conv = np.zeros_like(x)
    for ci, q, h, v in itertools.product(range(Ci), range(2), range(3), range(2)):
        conv[0, ci, q, h, v] = np.sum(w[ci] * y[0, :, 2 * q:2 * q + 2, 2 * h:2 * h + 2, 2 * v:2 * v + 2])
    assert abs(np.sum(up.a * y) - np.sum(x * conv)) < 1e-12
    np.testing.assert_allclose(orc.deconv2_bwd_data(Slab(y), w).a, conv, atol=1e-13)
    ones = orc.deconv2_fwd(Slab(np.ones((1, Ci, 2, 2, 2))), np.ones((Ci, Co, 2, 2, 2)), np.full(Co, 0.5))
    assert np.all(ones.a == Ci + 0.5)


def test_deconv_against_torch():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    Ci, Co = 3, 4
    x, w, b, g = rand(2, Ci, 2, 3, 2), rand(Ci, Co, 2, 2, 2), rand(Co), rand(2, Co, 4, 6, 4)
    tx, tw, tb = (torch.tensor(v, requires_grad=True) for v in (x, w, b))
    ty = F.conv_transpose3d(tx, tw, tb, stride=2)
    ty.backward(torch.tensor(g))
    np.testing.assert_allclose(orc.deconv2_fwd(Slab(x), w, b).a, ty.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(orc.deconv2_bwd_data(Slab(g), w).a, tx.grad.numpy(), atol=1e-13)
    dw, db = orc.deconv2_bwd_filter(Slab(x), Slab(g))
    np.testing.assert_allclose(dw, tw.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), atol=1e-12)


def test_concat_split():
    a, b = Slab(rand(1, 2, 3, 2, 2)), Slab(rand(1, 3, 3, 2, 2))
    c = orc.concat_c(a, b)
    assert np.array_equal(c.a[:, :2], a.a) and np.array_equal(c.a[:, 2:], b.a)
    ga, gb = orc.split_c(c, 2)
    assert np.array_equal(ga.a, a.a) and np.array_equal(gb.a, b.a)


# ---------------------------------------------------------------- dense + loss

def test_dense_and_mse_against_torch_and_finite_differences():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    x, w, b, t = rand(4, 7), rand(5, 7), rand(5), rand(4, 5)
    tx, tw, tb = (torch.tensor(v, requires_grad=True) for v in (x, w, b))
    ty = F.leaky_relu(F.linear(tx, tw, tb), 0.01)
    loss = F.mse_loss(ty, torch.tensor(t))
    loss.backward()
    y = orc.dense_fwd(x, w, b, orc.ACT_LEAKY, 0.01)
    L, dy = orc.mse_fwd_bwd(y, t)
    dx, dw, db = orc.dense_bwd(x, w, y, dy, orc.ACT_LEAKY, 0.01)
    assert abs(L - loss.item()) < 1e-14
    np.testing.assert_allclose(y, ty.detach().numpy(), atol=1e-14)
    np.testing.assert_allclose(dx, tx.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(dw, tw.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(db, tb.grad.numpy(), atol=1e-14)
    # closed form: pred = target + 1 everywhere -> loss 1, gradient 2/size
    L1, g1 = orc.mse_fwd_bwd(t + 1.0, t)
    assert abs(L1 - 1.0) < 1e-15 and np.allclose(g1, 2.0 / t.size)


def test_act_mask_bytes_of_a_hand_written_slab():
    """Sign mask of a saved activation (the (leaky-)ReLU derivative only needs z > 0): bytes written out by hand for two
    rows of 16 voxels inside a slab with one halo plane per side.  Bit k of byte j of a row is voxel 8 j + k, a zero and a
    negative zero are NOT positive, halo planes are left out, rows follow [n][c][interior plane][h]."""
    nz = -0.0
    assert np.signbit(nz)
    row0 = [1.0, -1.0, 0.0, nz, 2.0, 0.5, -3.0, 1e-30,      # bits 0,4,5,7      -> 0b10110001
            -2.0, 3.0, nz, 0.0, -1e-30, -5.0, 7.0, -0.25]   # bits 1,6          -> 0b01000010
    row1 = [-1.0, 1.0, 1.0, nz, 0.0, 0.0, 0.0, 3.0,         # bits 1,2,7        -> 0b10000110
            4.0, 4.0, 4.0, 4.0, 4.0, 4.0, 4.0, -4.0]        # bits 0..6         -> 0b01111111
    a = np.full((1, 1, 3, 2, 16), 9.0)                       # halo planes all positive: they must not show up
    a[0, 0, 1, 0], a[0, 0, 1, 1] = row0, row1
    m = orc.act_mask(Slab(a, 1, 1, 4, 12))
    assert m.dtype == np.uint8 and m.shape == (1, 1, 1, 2, 2)
    assert m.tolist() == [[[[[0b10110001, 0b01000010], [0b10000110, 0b01111111]]]]]
    # the same bytes by the definition, voxel by voxel (brute force over a seeded slab, several channels and planes)
    rng = np.random.default_rng(5)
    z = rng.standard_normal((2, 3, 4, 3, 24))
    z[rng.random(z.shape) < 0.2] = 0.0
    z[rng.random(z.shape) < 0.1] = nz
    got = orc.act_mask(Slab(z, 1, 0, 2, 8))
    for n, c, d, h, w in itertools.product(range(2), range(3), range(3), range(3), range(24)):
        assert (got[n, c, d, h, w // 8] >> (w % 8)) & 1 == (1 if z[n, c, d + 1, h, w] > 0 else 0)
