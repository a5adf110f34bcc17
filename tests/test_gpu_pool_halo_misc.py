"""GPU parity of pooling, halo pack/unpack (bit-exact), transposed conv, concat, dense and MSE."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED + 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [orc.POOL_AVG, orc.POOL_MAX])
@pytest.mark.parametrize("shape,halo", [((2, 3, 4, 6, 32), (0, 0)), ((1, 2, 6, 10, 12), (1, 1)),
                                        ((1, 5, 2, 4, 70), (2, 1)), ((1, 1, 8, 8, 2), (0, 0)),
                                        ((1, 16, 8, 32, 64), (1, 1))])
def test_pool_fwd_bwd(shape, halo, mode, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    a = synth.flat("normal", SEED, 1, (N, C, halo[0] + d + halo[1], H, W))
    if mode == orc.POOL_MAX:
        a = np.maximum(a, 0.0)          # post-ReLU input: all-zero windows make ties common
    xo, xg = slab_pair(a, dtype, halo, 4, 4 + d + 6)
    yo = orc.pool3d_fwd(xo, mode, y_halo=(1, 0))
    yg = dev_like(yo, dtype)
    h3d.pool3d_fwd(xg, yg, mode)
    got = from_dev(yg.t)
    if mode == orc.POOL_MAX:
        assert np.array_equal(got[:, :, 1:], yo.interior)
    else:
        close(got[:, :, 1:], yo.interior, (1e-6 if dtype == "f32" else 4e-3))
    assert np.all(got[:, :, 0] == 12345.0 if dtype == "f32" else got[:, :, 0] == quantize(12345.0, "bf16"))
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 2, yo.a.shape), dtype, (1, 0), yo.d_offset, yo.d_global)
    dxo = orc.pool3d_bwd(dyo, xo, mode, dx_halo=halo)
    dxg = h3d.Slab(torch.full(xo.a.shape, 7.0, dtype=xg.t.dtype, device="cuda"), halo[0], halo[1], xo.d_offset, xo.d_global)
    h3d.pool3d_bwd(dyg, xg if mode == orc.POOL_MAX else None, dxg, mode)
    got = from_dev(dxg.interior)
    if mode == orc.POOL_MAX:
        assert np.array_equal(got, dxo.interior)     # routing is exact, ties included
    else:
        close(got, dxo.interior, (1e-6 if dtype == "f32" else 4e-3))
    if halo[0]:
        assert np.all(from_dev(dxg.t)[:, :, :halo[0]] == 7.0)


def test_pool_rejects_odd_extents():
    import torch
    import paper_2007_12856_amd as h3d
    x = h3d.Slab(torch.zeros((1, 1, 3, 4, 4), device="cuda"))
    y = h3d.Slab(torch.zeros((1, 1, 1, 2, 2), device="cuda"))
    with pytest.raises(h3d.H3DError) as e:
        h3d.pool3d_fwd(x, y, h3d.POOL_AVG)
    assert e.value.status == -2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 4, 4, 5), (1, 4, 6, 16, 32), (1, 1, 2, 3, 3)])
def test_halo_exchange_is_bit_exact(shape, dtype):
    """Three shards of one volume on one GPU exchange faces: pack the neighbour's edge, unpack into
    the halo (zero fill at the global boundary).  Every byte must equal the full volume's."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    Dg = 3 * d
    full = quantize(synth.flat("normal", SEED, 3, (N, C, Dg, H, W)), dtype)
    for width in (1, 2):
        if width > d:
            continue
        shards_o, shards_g = [], []
        for s in range(3):
            a = np.full((N, C, d + 4, H, W), 777.0)
            a[:, :, 2:2 + d] = full[:, :, s * d:(s + 1) * d]
            o, g = slab_pair(a, dtype, (2, 2), s * d, Dg)
            shards_o.append(o)
            shards_g.append(g)
        for s in range(3):
            for face, nb, nb_face in ((orc.FACE_D_LO, s - 1, orc.FACE_D_HI), (orc.FACE_D_HI, s + 1, orc.FACE_D_LO)):
                if 0 <= nb < 3:
                    bo = orc.halo_pack(shards_o[nb], nb_face, width)
                    nbytes = h3d.halo_bytes(shards_g[nb], width)
                    assert nbytes == bo.size * (4 if dtype == "f32" else 2)
                    bg = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
                    h3d.halo_pack(shards_g[nb], nb_face, width, bg)
                    view = bg.view(torch.float32 if dtype == "f32" else torch.bfloat16).view(bo.shape)
                    assert np.array_equal(from_dev(view), bo)
                    orc.halo_unpack(bo, shards_o[s], face, width)
                    h3d.halo_unpack(bg, shards_g[s], face, width)
                else:
                    orc.halo_unpack(None, shards_o[s], face, width)
                    h3d.halo_unpack(None, shards_g[s], face, width)
        for s in range(3):
            assert np.array_equal(from_dev(shards_g[s].t), shards_o[s].a)   # canaries included


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,halo", [((2, 3, 4, 4, 5), (2, 2)), ((1, 4, 6, 16, 32), (1, 2)), ((1, 1, 2, 3, 3), (2, 1)),
                                        ((2, 16, 8, 32, 64), (1, 1))])
def test_both_faces_in_one_call_equal_the_two_calls(shape, halo, dtype):
    """FACE_D_BOTH packs / unpacks the two depth faces with one launch: the buffer is the LO face followed by the HI
    face, each bit for bit what the oracle's per-face call gives; NULL zero-fills both halos; canary planes stay."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    a = synth.flat("normal", SEED, 23, (N, C, halo[0] + d + halo[1], H, W))
    for width in (1, 2):
        if width > d:
            continue
        o, g = slab_pair(a, dtype, halo, 8, 8 + d + 8)
        k = h3d.halo_bytes(g, width) // (4 if dtype == "f32" else 2)
        buf = torch.full((2 * k,), 5.0, dtype=tdt, device="cuda")
        h3d.halo_pack(g, h3d.FACE_D_BOTH, width, buf)
        lo, hi = orc.halo_pack(o, orc.FACE_D_LO, width), orc.halo_pack(o, orc.FACE_D_HI, width)
        assert np.array_equal(from_dev(buf[:k]).reshape(lo.shape), lo) and np.array_equal(from_dev(buf[k:]).reshape(hi.shape), hi)
        if width > min(halo):
            with pytest.raises(h3d.H3DError) as e:
                h3d.halo_unpack(buf, g, h3d.FACE_D_BOTH, width)
            assert e.value.status == -4
            continue
        # unpack what was packed, swapped as two neighbours of the same content would send it
        sw = torch.cat([buf[k:], buf[:k]])
        h3d.halo_unpack(sw, g, h3d.FACE_D_BOTH, width)
        orc.halo_unpack(hi, o, orc.FACE_D_LO, width)
        orc.halo_unpack(lo, o, orc.FACE_D_HI, width)
        assert np.array_equal(from_dev(g.t), o.a)
        h3d.halo_unpack(None, g, h3d.FACE_D_BOTH, width)
        orc.halo_unpack(None, o, orc.FACE_D_LO, width)
        orc.halo_unpack(None, o, orc.FACE_D_HI, width)
        assert np.array_equal(from_dev(g.t), o.a)
    with pytest.raises(h3d.H3DError) as e:
        h3d.halo_pack(g, 3, 1, buf)
    assert e.value.status == -1


# (N, C, D, H, W) stored extents and boxes (d0, h0, w0, bd, bh, bw): D, H and W faces one and two voxels wide, at both
# ends, aligned and unaligned, a whole-tensor box, a single element, an empty box
BOX_CASES = [
    ((2, 3, 6, 10, 32), [(0, 0, 0, 1, 10, 32), (4, 0, 0, 2, 10, 32), (0, 0, 0, 6, 1, 32), (0, 8, 0, 6, 2, 32),
                         (0, 0, 0, 6, 10, 1), (0, 0, 30, 6, 10, 2), (1, 1, 8, 4, 8, 16), (0, 0, 0, 6, 10, 32)]),
    ((1, 5, 3, 7, 9), [(0, 0, 0, 3, 7, 1), (0, 0, 7, 3, 7, 2), (0, 6, 0, 3, 1, 9), (2, 0, 0, 1, 7, 9), (1, 3, 4, 1, 1, 1),
                       (0, 0, 0, 0, 7, 9)]),
    ((1, 2, 4, 4, 70), [(0, 0, 1, 4, 4, 68), (0, 3, 0, 4, 1, 70), (0, 0, 68, 4, 4, 2)]),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,boxes", BOX_CASES)
def test_general_faces_are_bit_exact(shape, boxes, dtype):
    """H and W faces (and any other box) packed and unpacked on the GPU equal the oracle's bytes; elements outside the
    box keep their canary; a NULL buffer zero-fills."""
    import torch
    import paper_2007_12856_amd as h3d
    a = quantize(synth.flat("normal", SEED, 30, shape), dtype)
    tg = to_dev(a, dtype)
    for box in boxes:
        bo = orc.box_pack(a, box)
        nbytes = h3d.box_bytes(tg, box)
        assert nbytes == bo.size * (4 if dtype == "f32" else 2)
        bg = torch.full(bo.shape, 3.0, dtype=tg.dtype, device="cuda")
        h3d.box_pack(tg, box, bg)
        assert np.array_equal(from_dev(bg), bo)
        uo = np.full(shape, quantize(777.0, dtype))
        ug = to_dev(uo, dtype)
        orc.box_unpack(bo, uo, box)
        h3d.box_unpack(bg, ug, box)
        assert np.array_equal(from_dev(ug), uo)
        orc.box_unpack(None, uo, box)
        h3d.box_unpack(None, ug, box)
        assert np.array_equal(from_dev(ug), uo)


def test_box_errors():
    import torch
    import paper_2007_12856_amd as h3d
    t = torch.zeros((1, 1, 4, 4, 8), device="cuda")
    buf = torch.zeros(256, device="cuda")
    for box in [(0, 0, 7, 4, 4, 2), (-1, 0, 0, 1, 4, 8), (0, 3, 0, 4, 2, 8)]:
        with pytest.raises(h3d.H3DError) as e:
            h3d.box_pack(t, box, buf)
        assert e.value.status == -1


def test_halo_width_errors():
    import torch
    import paper_2007_12856_amd as h3d
    t = h3d.Slab(torch.zeros((1, 1, 4, 2, 2), device="cuda"), 1, 1)
    buf = torch.zeros(64, device="cuda")
    with pytest.raises(h3d.H3DError) as e:
        h3d.halo_unpack(buf, t, h3d.FACE_D_LO, 2)
    assert e.value.status == -4
    with pytest.raises(h3d.H3DError) as e:
        h3d.halo_pack(t, h3d.FACE_D_LO, 3, buf)
    assert e.value.status == -1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cin,cout,shape", [(3, 5, (2, 2, 3, 5)), (16, 8, (1, 4, 6, 34)), (128, 64, (1, 2, 4, 16)),
                                            (40, 24, (2, 3, 5, 40)), (20, 70, (1, 2, 9, 64)), (136, 16, (1, 1, 4, 32)),
                                            (48, 40, (1, 2, 3, 24)), (100, 21, (1, 1, 2, 16))])
def test_deconv2(cin, cout, shape, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, d, H, W = shape
    b = np.sqrt(3.0 / (8 * cin))
    w = quantize(synth.flat("uniform", SEED, 4, (cin, cout, 2, 2, 2), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, 5, (cout,), -0.1, 0.1)).astype(np.float64)
    xo, xg = slab_pair(synth.flat("normal", SEED, 6, (N, cin, d, H, W)), dtype, (0, 0), 2, 2 + d + 2)
    yo = orc.deconv2_fwd(xo, w, bias)
    yg = h3d.deconv2_fwd(xg, to_dev(w, dtype), to_dev(bias, "f32"), dev_like(yo, dtype))
    close(from_dev(yg.t), yo.a, TOL[dtype])
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 7, yo.a.shape), dtype, (0, 0), yo.d_offset, yo.d_global)
    dxo = orc.deconv2_bwd_data(dyo, w)
    dxg = h3d.deconv2_bwd_data(dyg, to_dev(w, dtype), dev_like(dxo, dtype))
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.deconv2_bwd_filter(xo, dyo)
    dw = torch.empty((cin, cout, 2, 2, 2), device="cuda")
    db = torch.empty((cout,), device="cuda")
    h3d.deconv2_bwd_filter(xg, dyg, dw, db)
    close(from_dev(dw), dwo, TOL[dtype])
    close(from_dev(db), dbo, TOL[dtype])
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.deconv2_bwd_filter(xg, dyg, dw2, db2)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_concat_split_bit_exact(dtype):
    import paper_2007_12856_amd as h3d
    ao, ag = slab_pair(synth.flat("normal", SEED, 8, (2, 3, 6, 5, 7)), dtype, (1, 1), 4, 12)
    bo, bg = slab_pair(synth.flat("normal", SEED, 9, (2, 5, 4, 5, 7)), dtype, (0, 0), 4, 12)
    co = orc.concat_c(ao, bo)
    cg = h3d.concat_c(ag, bg, dev_like(co, dtype))
    assert np.array_equal(from_dev(cg.t), co.a)
    a2, b2 = dev_like(orc.Slab(ao.interior, 0, 0, 4, 12), dtype), dev_like(bo, dtype)
    h3d.split_c(cg, a2, b2)
    assert np.array_equal(from_dev(a2.t), ao.interior) and np.array_equal(from_dev(b2.t), bo.a)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m,n,k,act", [(4, 64, 512, orc.ACT_LEAKY), (3, 7, 33, orc.ACT_NONE), (8, 300, 1000, orc.ACT_RELU),
                                       (4, 4, 256, orc.ACT_NONE), (1, 130, 2048, orc.ACT_LEAKY),
                                       (4, 2048, 1024, orc.ACT_LEAKY), (4, 1032, 2080, orc.ACT_LEAKY), (8, 1024, 4096, orc.ACT_NONE),
                                       (4, 300, 4096, orc.ACT_LEAKY), (3, 2048, 8192, orc.ACT_NONE), (2, 256, 12288, orc.ACT_RELU),
                                       (4, 4100, 4096, orc.ACT_LEAKY)])
def test_dense_and_mse(m, n, k, act, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    b = np.sqrt(3.0 / k)
    x = quantize(synth.flat("normal", SEED, 10, (m, k)), dtype)
    w = quantize(synth.flat("uniform", SEED, 11, (n, k), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, 12, (n,), -0.1, 0.1)).astype(np.float64)
    yo = orc.dense_fwd(x, w, bias, act, 0.01)
    y = torch.empty((m, n), dtype=td, device="cuda")
    h3d.dense_fwd(to_dev(x, dtype), to_dev(w, dtype), to_dev(bias, "f32"), y, act, 0.01)
    close(from_dev(y), yo, TOL[dtype])
    yq = quantize(yo, dtype)
    dy = quantize(synth.flat("normal", SEED, 13, (m, n)), dtype)
    dxo, dwo, dbo = orc.dense_bwd(x, w, yq, dy, act, 0.01)
    dx = torch.empty((m, k), dtype=td, device="cuda")
    dw = torch.empty((n, k), device="cuda")
    db = torch.empty((n,), device="cuda")
    h3d.dense_bwd(to_dev(x, dtype), to_dev(w, dtype), to_dev(yq, dtype), to_dev(dy, dtype), dx, dw, db, act, 0.01)
    close(from_dev(dx), dxo, TOL[dtype])
    close(from_dev(dw), dwo, TOL[dtype])
    close(from_dev(db), dbo, TOL[dtype])
    # the two halves asked for separately (a caller may put them on two streams): same bits
    dx2, dw2, db2 = torch.full_like(dx, 3.0), torch.full_like(dw, 3.0), torch.full_like(db, 3.0)
    args = (to_dev(x, dtype), to_dev(w, dtype), to_dev(yq, dtype), to_dev(dy, dtype))
    h3d.dense_bwd(*args, dx2, None, None, act, 0.01)
    h3d.dense_bwd(*args, None, dw2, db2, act, 0.01)
    assert torch.equal(dx, dx2) and torch.equal(dw, dw2) and torch.equal(db, db2)
    # loss
    t = synth.round_f32(synth.flat("uniform", SEED, 14, (m, n))).astype(np.float64)
    Lo, go = orc.mse_fwd_bwd(yq, t)
    loss = torch.empty((1,), device="cuda")
    dp = torch.empty((m, n), dtype=td, device="cuda")
    h3d.mse_fwd_bwd(to_dev(yq, dtype), to_dev(t, "f32"), loss, dp)
    assert abs(loss.item() - Lo) <= 1e-5 * abs(Lo)
    close(from_dev(dp), go, TOL[dtype])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 4, 5, 7), (1, 8, 4, 6, 16)])
def test_act_bwd(shape, dtype):
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 20, (N, C, d + 2, H, W)), dtype, (1, 1), 4, 16)
    d2o, d2g = slab_pair(synth.flat("normal", SEED, 21, (N, C, d, H, W)), dtype, (0, 0), 4, 16)
    zo, zg = slab_pair(synth.flat("normal", SEED, 22, (N, C, d + 1, H, W)), dtype, (0, 1), 4, 16)
    for act, two in [(orc.ACT_LEAKY, False), (orc.ACT_RELU, True), (orc.ACT_NONE, True)]:
        go = orc.act_bwd(dzo, d2o if two else None, zo, act, 0.01, g_halo=(2, 0))
        gg = dev_like(go, dtype)
        h3d.act_bwd(dzg, d2g if two else None, zg, gg, act, 0.01)
        got = from_dev(gg.t)
        close(got[:, :, 2:], go.interior, (1e-6 if dtype == "f32" else 4e-3))
        assert np.all(got[:, :, :2] == quantize(12345.0, dtype))      # halo planes untouched


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [orc.POOL_AVG, orc.POOL_MAX])
def test_pool_bwd_fused_with_activation_backward(mode, dtype):
    """g = pool_bwd(dy) * act'(z) in one pass equals the two oracle steps (one rounding of g)."""
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = 2, 3, 4, 6, 16
    xo, xg = slab_pair(np.maximum(synth.flat("normal", SEED, 30, (N, C, d, H, W)), 0), dtype, (0, 0), 8, 32)
    zo, zg = slab_pair(synth.flat("normal", SEED, 31, (N, C, d + 2, H, W)), dtype, (1, 1), 8, 32)
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 32, (N, C, d // 2, H // 2, W // 2)), dtype, (0, 0), 4, 16)
    for act in (orc.ACT_LEAKY, orc.ACT_RELU):
        ref = orc.act_bwd(orc.pool3d_bwd(dyo, xo, mode), None, zo, act, 0.01)
        gg = dev_like(ref, dtype)
        h3d.pool3d_bwd_act(dyg, xg if mode == orc.POOL_MAX else None, zg, gg, mode, act, 0.01)
        close(from_dev(gg.t), ref.a, (1e-6 if dtype == "f32" else 4e-3))


# ---------------------------------------------------------------- views: channel ranges / plane runs of a larger tensor
def _parent(shape, halo, seed_stream, fill=None):
    """a packed device slab of noise (or a constant) whose channel ranges / plane runs serve as views"""
    import torch
    import paper_2007_12856_amd as h3d
    a = synth.flat("normal", SEED, seed_stream, shape) if fill is None else np.full(shape, fill)
    return a, h3d.Slab(to_dev(quantize(a, "bf16"), "bf16"), halo, halo, 4, 4 + shape[2] - 2 * halo + 6)


@pytest.mark.parametrize("mode", ["avg", "max"])
def test_pool_act_and_skip_add_on_channel_views(mode):
    """The U-Net level's zero-copy concatenation: pooling forward reads one half of a 2C-channel slab in place, the fused
    pooling backward reads the saved activation and the skip gradient as halves of two other slabs and adds the skip
    gradient before the activation derivative; results equal the oracle's composition and, bit for bit, the same calls
    on packed copies; nothing outside the addressed halves is touched."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = 2, 3, 4, 6, 32
    code = h3d.POOL_AVG if mode == "avg" else h3d.POOL_MAX
    ocode = orc.POOL_AVG if mode == "avg" else orc.POOL_MAX
    za, zp = _parent((N, 2 * C, d + 2, H, W), 1, 61)             # the "cat" slab (1-plane halo): the skip half is channels [0, C)
    za[:, :, :, 0] = 0.0                                          # ties after ReLU
    zp.t.copy_(to_dev(quantize(za, "bf16"), "bf16"))
    da, dp_ = _parent((N, 2 * C, d, H, W), 0, 62)                 # the "dcat" slab: the skip gradient is channels [0, C)
    zv, skipv = zp.channels(0, C, 0, 0), dp_.channels(0, C)
    zq = quantize(za, "bf16")[:, :C, 1:-1]
    skipq = quantize(da, "bf16")[:, :C]
    zo = orc.Slab(zq, 0, 0, 4, zp.d_global)
    # forward on the view
    yo = orc.pool3d_fwd(zo, ocode)
    yg = dev_like(yo, "bf16")
    h3d.pool3d_fwd(zv, yg, code)
    yc = dev_like(yo, "bf16")
    h3d.pool3d_fwd(h3d.Slab(zv.t.contiguous(), 0, 0, 4, zp.d_global), yc, code)
    assert torch.equal(yg.t, yc.t)
    close(from_dev(yg.t), yo.a, 4e-3, "pooled view")
    # backward: g = (pool_bwd(dy) + skip) * relu'(z), written into a slab with a halo
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 63, (N, C, d // 2, H // 2, W // 2)), "bf16", (0, 0), 2, zp.d_global // 2)
    g = h3d.Slab(torch.full((N, C, d + 2, H, W), 7.0, dtype=torch.bfloat16, device="cuda"), 1, 1, 4, zp.d_global)
    h3d.pool3d_bwd_act(dyg, zv, zv, g, code, h3d.ACT_RELU, 0.0, dz2=skipv)
    un = quantize(orc.pool3d_bwd(dyo, zo, ocode).a, "bf16")       # the un-pooled gradient as pool3d_bwd stores it
    want = (un + skipq) * (zq > 0)
    close(from_dev(g.interior), want, 4e-3, "fused pooling backward", elem=2.0 ** -8)
    assert bool((g.t[:, :, [0, -1]] == 7.0).all())
    # the separate calls on packed copies: same bits
    zc = h3d.Slab(zv.t.contiguous(), 0, 0, 4, zp.d_global)
    d1 = h3d.Slab(torch.empty((N, C, d, H, W), dtype=torch.bfloat16, device="cuda"), 0, 0, 4, zp.d_global)
    h3d.pool3d_bwd(dyg, zc, d1, code)
    g2 = h3d.Slab(torch.empty((N, C, d, H, W), dtype=torch.bfloat16, device="cuda"), 0, 0, 4, zp.d_global)
    h3d.act_bwd(d1, h3d.Slab(skipv.t.contiguous(), 0, 0, 4, zp.d_global), zc, g2, h3d.ACT_RELU)
    assert torch.equal(g.interior, g2.t)
    # act_bwd itself on views (z and the second gradient in place)
    g3 = h3d.Slab(torch.empty((N, C, d, H, W), dtype=torch.bfloat16, device="cuda"), 0, 0, 4, zp.d_global)
    h3d.act_bwd(d1, skipv, zv, g3, h3d.ACT_RELU)
    assert torch.equal(g3.t, g2.t)
    # the parents are unchanged
    assert torch.equal(zp.t, to_dev(quantize(za, "bf16"), "bf16")) and torch.equal(dp_.t, to_dev(quantize(da, "bf16"), "bf16"))


def test_deconv_writes_and_reads_channel_views():
    """Transposed convolution straight into the upper half of a 2C-channel slab with a halo, and its two backward passes
    reading the upper half of the gradient slab in place: same bits as on packed tensors, the other half and the halo
    planes untouched."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, dc, Hc, Wc = 1, 32, 16, 3, 6, 16
    b = np.sqrt(3.0 / (8 * Ci))
    w = quantize(synth.flat("uniform", SEED, 71, (Ci, Co, 2, 2, 2), -b, b), "bf16")
    bias = synth.round_f32(synth.flat("uniform", SEED, 72, (Co,), -0.1, 0.1)).astype(np.float64)
    xo, xg = slab_pair(synth.flat("normal", SEED, 73, (N, Ci, dc, Hc, Wc)), "bf16", (0, 0), 2, 8)
    wd, bd = to_dev(w, "bf16"), to_dev(bias, "f32")
    cat = h3d.Slab(torch.full((N, 2 * Co, 2 * dc + 2, 2 * Hc, 2 * Wc), 5.0, dtype=torch.bfloat16, device="cuda"), 1, 1, 4, 16)
    up = cat.channels(Co, 2 * Co, 0, 0)
    h3d.deconv2_fwd(xg, wd, bd, up)
    yc = h3d.Slab(torch.empty((N, Co, 2 * dc, 2 * Hc, 2 * Wc), dtype=torch.bfloat16, device="cuda"), 0, 0, 4, 16)
    h3d.deconv2_fwd(xg, wd, bd, yc)
    assert torch.equal(up.t, yc.t)
    assert bool((cat.t[:, :Co] == 5.0).all()) and bool((cat.t[:, :, [0, -1]] == 5.0).all())
    close(from_dev(up.t), orc.deconv2_fwd(xo, w, bias).a, TOL["bf16"], "deconv into a view")
    dcat = h3d.Slab(to_dev(quantize(synth.flat("normal", SEED, 74, (N, 2 * Co, 2 * dc, 2 * Hc, 2 * Wc)), "bf16"), "bf16"), 0, 0, 4, 16)
    dup = dcat.channels(Co, 2 * Co)
    dupc = h3d.Slab(dup.t.contiguous(), 0, 0, 4, 16)
    dx1, dx2 = dev_like(xo, "bf16"), dev_like(xo, "bf16")
    h3d.deconv2_bwd_data(dup, wd, dx1)
    h3d.deconv2_bwd_data(dupc, wd, dx2)
    assert torch.equal(dx1.t, dx2.t)
    dw1, db1 = torch.empty((Ci, Co, 2, 2, 2), device="cuda"), torch.empty((Co,), device="cuda")
    dw2, db2 = torch.empty_like(dw1), torch.empty_like(db1)
    h3d.deconv2_bwd_filter(xg, dup, dw1, db1)
    h3d.deconv2_bwd_filter(xg, dupc, dw2, db2)
    assert torch.equal(dw1, dw2) and torch.equal(db1, db2)
    dwo, dbo = orc.deconv2_bwd_filter(xo, orc.Slab(from_dev(dupc.t), 0, 0, 4, 16))
    close(from_dev(dw1), dwo, 2e-4, "deconv dw from a view")
