"""GPU parity of the stride-2 3x3x3 convolution (Table I, fourth convolution) against the CPU oracle:
all three passes, unsharded and on depth shards with the halo sides each direction needs, fp32 and bf16,
odd H / W, channel counts that divide nothing, canaries on what must not be written."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, cut, dev_like, elem_masked_bf, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED

# (N, Cin, Cout, Dg, H, W)
SHAPES = [
    (1, 64, 128, 8, 8, 8),       # the layer's channel counts on a small volume
    (2, 3, 5, 4, 7, 9),          # odd H and W, nothing divides anything
    (1, 16, 32, 6, 12, 40),
    (1, 8, 16, 2, 2, 2),         # a single output voxel
    (1, 4, 16, 4, 16, 64),
]


def _weights(cin, cout, dtype, stream):
    b = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, stream, (cout, cin, 3, 3, 3), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, stream + 1, (cout,), -0.1, 0.1)).astype(np.float64)
    return w, bias


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_stride2_three_passes_unsharded(shape, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = shape
    alpha = 0.01
    w, bias = _weights(Ci, Co, dtype, 310)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    xo, xg = slab_pair(synth.flat("uniform", SEED, 301, (N, Ci, D, H, W)), dtype)
    yo = orc.conv3d_s2_fwd(xo, w, bias, orc.ACT_LEAKY, alpha)
    yg = h3d.conv3d_s2_fwd(xg, wd, bd, dev_like(yo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(yg.t), yo.a, TOL[dtype])
    yq_o, yq_g = slab_pair(yo.a, dtype)
    dyo, dyg = slab_pair(synth.flat("uniform", SEED, 302, yo.a.shape), dtype)
    dxo = orc.conv3d_s2_bwd_data(dyo, yq_o, w, xo, orc.ACT_LEAKY, alpha)
    dxg = h3d.conv3d_s2_bwd_data(dyg, yq_g, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.conv3d_s2_bwd_filter(xo, dyo, yq_o, orc.ACT_LEAKY, alpha)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_s2_bwd_filter(xg, dyg, yq_g, dw, db, h3d.ACT_LEAKY, alpha)
    tol_w = 1e-5 if dtype == "f32" else 2e-4
    close(from_dev(dw), dwo, tol_w, elem=elem_masked_bf(dtype))
    close(from_dev(db), dbo, tol_w, elem=elem_masked_bf(dtype))
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_s2_bwd_filter(xg, dyg, yq_g, dw2, db2, h3d.ACT_LEAKY, alpha)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_RELU])
def test_stride2_no_bias_other_activations(dtype, act):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = 1, 8, 16, 4, 6, 20
    w, _ = _weights(Ci, Co, dtype, 320)
    wd = to_dev(w, dtype)
    xo, xg = slab_pair(synth.flat("normal", SEED, 303, (N, Ci, D, H, W)), dtype)
    yo = orc.conv3d_s2_fwd(xo, w, None, act)
    yg = h3d.conv3d_s2_fwd(xg, wd, None, dev_like(yo, dtype), act, 0.0)
    close(from_dev(yg.t), yo.a, TOL[dtype])
    yq_o, yq_g = slab_pair(yo.a, dtype)
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 304, yo.a.shape), dtype)
    dxo = orc.conv3d_s2_bwd_data(dyo, yq_o, w, xo, act)
    dxg = h3d.conv3d_s2_bwd_data(dyg, yq_g, wd, dev_like(dxo, dtype), act, 0.0)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, _ = orc.conv3d_s2_bwd_filter(xo, dyo, yq_o, act)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    h3d.conv3d_s2_bwd_filter(xg, dyg, yq_g, dw, None, act, 0.0)
    close(from_dev(dw), dwo, (1e-5 if dtype == "f32" else 2e-4))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shard", [0, 1, 3])
def test_stride2_on_depth_shards(shard, dtype):
    """4-way depth partition of a 1 x 8 x 16 x 10 x 24 sample: forward and backward-filter read the lower halo
    of x, backward-data the upper halo of dy and y; outputs carry halos that must stay untouched."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, Dg, H, W = 1, 8, 16, 16, 10, 24
    d, alpha = Dg // 4, 0.01
    off = shard * d
    w, bias = _weights(Ci, Co, dtype, 330)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    full_x = (N, Ci, Dg, H, W)
    full_y = (N, Co, Dg // 2, H // 2, W // 2)
    # forward: x with halo 1/1 (the upper one is never read: poison it), y with halos 1/1 holding canaries
    xa = cut("uniform", SEED, 305, full_x, off, d, (1, 1))
    xa[:, :, -1] = np.nan
    xo, xg = slab_pair(xa, dtype, (1, 1), off, Dg)
    yo = orc.conv3d_s2_fwd(xo, w, bias, orc.ACT_LEAKY, alpha)
    yg = h3d.Slab(torch.full((N, Co, d // 2 + 2, H // 2, W // 2), 12345.0, device="cuda",
                             dtype=torch.float32 if dtype == "f32" else torch.bfloat16), 1, 1, off // 2, Dg // 2)
    h3d.conv3d_s2_fwd(xg, wd, bd, yg, h3d.ACT_LEAKY, alpha)
    got = from_dev(yg.t)
    close(got[:, :, 1:-1], yo.a, TOL[dtype])
    assert np.all(got[:, :, 0] == from_dev(torch.full((1,), 12345.0, device="cuda", dtype=yg.t.dtype))[0])
    assert np.all(got[:, :, -1] == got[0, 0, 0, 0, 0])
    # backward: dy and the saved y with halo 0/1 cut from the seeded full tensors; lower halos absent
    dya = cut("uniform", SEED, 306, full_y, off // 2, d // 2, (0, 1))
    ya = cut("normal", SEED, 307, full_y, off // 2, d // 2, (0, 1))
    dyo, dyg = slab_pair(dya, dtype, (0, 1), off // 2, Dg // 2)
    yso, ysg = slab_pair(ya, dtype, (0, 1), off // 2, Dg // 2)
    xin = orc.Slab(xo.interior, 0, 0, off, Dg)
    dxo = orc.conv3d_s2_bwd_data(dyo, yso, w, xin, orc.ACT_LEAKY, alpha)
    dxg = h3d.conv3d_s2_bwd_data(dyg, ysg, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.conv3d_s2_bwd_filter(xo, dyo, yso, orc.ACT_LEAKY, alpha)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_s2_bwd_filter(xg, dyg, ysg, dw, db, h3d.ACT_LEAKY, alpha)
    tol_w = 1e-5 if dtype == "f32" else 2e-4
    close(from_dev(dw), dwo, tol_w, elem=elem_masked_bf(dtype))
    close(from_dev(db), dbo, tol_w, elem=elem_masked_bf(dtype))


def test_stride2_errors_do_not_launch():
    import ctypes
    import torch
    import paper_2007_12856_amd as h3d
    w = torch.zeros((3, 2, 3, 3, 3), device="cuda")
    x = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda"), 0, 0, 4, 16)       # interior shard, no lower halo
    y = h3d.Slab(torch.zeros((1, 3, 2, 2, 2), device="cuda"), 0, 0, 2, 8)
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_s2_fwd(x, w, None, y)
    assert e.value.status == -4
    with pytest.raises(h3d.H3DError) as e:                                       # dy without its upper halo
        h3d.conv3d_s2_bwd_data(y, None, w, x)
    assert e.value.status == -4
    xodd = h3d.Slab(torch.zeros((1, 2, 3, 4, 4), device="cuda"))
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_s2_fwd(xodd, w, None, h3d.Slab(torch.zeros((1, 3, 1, 2, 2), device="cuda")))
    assert e.value.status == -2
    xs = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda"))
    with pytest.raises(h3d.H3DError) as e:                                       # wrong output extents
        h3d.conv3d_s2_fwd(xs, w, None, h3d.Slab(torch.zeros((1, 3, 2, 2, 3), device="cuda")))
    assert e.value.status == -1
    ys = h3d.Slab(torch.zeros((1, 3, 2, 2, 2), device="cuda"))
    st = h3d.lib().h3d_conv3d_s2_fwd(h3d.handle(), ctypes.byref(xs.desc()), ctypes.c_void_p(w.data_ptr()), None,
                                     ctypes.byref(ys.desc()), 0, 0.0, None, 0, None)
    assert st == -3


def test_stride2_empty_shard():
    import torch
    import paper_2007_12856_amd as h3d
    x = h3d.Slab(torch.zeros((1, 2, 0, 4, 4), device="cuda"), 0, 0, 0, 8)
    y = h3d.Slab(torch.zeros((1, 3, 0, 2, 2), device="cuda"), 0, 0, 0, 4)
    w = torch.zeros((3, 2, 3, 3, 3), device="cuda")
    h3d.conv3d_s2_fwd(x, w, None, y)
    dw = torch.full((3, 2, 3, 3, 3), 5.0, device="cuda")
    h3d.conv3d_s2_bwd_filter(x, y, None, dw, None)
    torch.cuda.synchronize()
    assert float(dw.abs().max()) == 0.0
