"""GPU parity of the 5x5x5 convolution (Sec. III-A: 3^3 and 5^3 filters; two halo planes) against the CPU oracle:
all three passes, unsharded and on depth shards with two halo planes, fp32 and bf16, extents that span several
8 x 32 tiles with ragged tails, channel counts on both sides of the 16-channel blocks, canaries on what must not
be written, error paths that must not launch."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, cut, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED

# (N, Cin, Cout, D, H, W)
SHAPES = [
    (1, 1, 1, 1, 1, 1),          # a single voxel: only the centre tap is inside the volume
    (2, 3, 5, 4, 11, 37),        # ragged tiles in both directions
    (1, 16, 32, 6, 16, 64),      # two channel blocks, whole tiles
    (1, 17, 18, 3, 9, 33),       # one channel past a block on both sides
    (1, 4, 16, 5, 20, 70),
    (1, 33, 34, 2, 35, 136),     # two tiles in H and in W for every kernel form, one channel past a 32-block
]


def _weights(cin, cout, dtype, stream):
    b = np.sqrt(3.0 / (125 * cin))
    w = quantize(synth.flat("uniform", SEED, stream, (cout, cin, 5, 5, 5), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, stream + 1, (cout,), -0.1, 0.1)).astype(np.float64)
    return w, bias


def _tol_w(dtype):
    return 1e-5 if dtype == "f32" else 2e-4


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_k5_three_passes_unsharded(shape, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = shape
    alpha = 0.01
    print("k5 unsharded", shape, dtype, flush=True)
    w, bias = _weights(Ci, Co, dtype, 510)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    xo, xg = slab_pair(synth.flat("uniform", SEED, 501, (N, Ci, D, H, W)), dtype)
    zo = orc.convk_fwd(xo, w, bias, orc.ACT_LEAKY, alpha)
    zg = h3d.conv3d_k5_fwd(xg, wd, bd, dev_like(zo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(zg.t), zo.a, TOL[dtype])
    zq_o, zq_g = slab_pair(zo.a, dtype)
    dzo, dzg = slab_pair(synth.flat("uniform", SEED, 502, zo.a.shape), dtype)
    dxo = orc.convk_bwd_data(dzo, zq_o, w, orc.ACT_LEAKY, alpha)
    dxg = h3d.conv3d_k5_bwd_data(dzg, zq_g, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.convk_bwd_filter(5, xo, dzo, zq_o, orc.ACT_LEAKY, alpha)
    dw = torch.full((Co, Ci, 5, 5, 5), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_k5_bwd_filter(xg, dzg, zq_g, dw, db, h3d.ACT_LEAKY, alpha)
    close(from_dev(dw), dwo, _tol_w(dtype))
    close(from_dev(db), dbo, _tol_w(dtype))
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_k5_bwd_filter(xg, dzg, zq_g, dw2, db2, h3d.ACT_LEAKY, alpha)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_RELU])
def test_k5_no_bias_other_activations(dtype, act):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = 1, 8, 16, 4, 6, 20
    print("k5 act", act, dtype, flush=True)
    w, _ = _weights(Ci, Co, dtype, 520)
    wd = to_dev(w, dtype)
    xo, xg = slab_pair(synth.flat("normal", SEED, 503, (N, Ci, D, H, W)), dtype)
    zo = orc.convk_fwd(xo, w, None, act)
    zg = h3d.conv3d_k5_fwd(xg, wd, None, dev_like(zo, dtype), act, 0.0)
    close(from_dev(zg.t), zo.a, TOL[dtype])
    zq_o, zq_g = slab_pair(zo.a, dtype)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 504, zo.a.shape), dtype)
    dxo = orc.convk_bwd_data(dzo, zq_o, w, act)
    dxg = h3d.conv3d_k5_bwd_data(dzg, zq_g, wd, dev_like(dxo, dtype), act, 0.0)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, _ = orc.convk_bwd_filter(5, xo, dzo, zq_o, act)
    dw = torch.full((Co, Ci, 5, 5, 5), 777.0, device="cuda")
    h3d.conv3d_k5_bwd_filter(xg, dzg, zq_g, dw, None, act, 0.0)
    close(from_dev(dw), dwo, _tol_w(dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shard", [0, 1, 3])
def test_k5_on_depth_shards(shard, dtype):
    """4-way depth partition of a 1 x 6 x 12 x 10 x 40 sample, two halo planes per side (zeros outside the volume):
    each shard's result is the oracle's on the same shard; outputs carry halos that must stay untouched."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, Dg, H, W = 1, 6, 20, 12, 10, 40
    d, alpha = Dg // 4, 0.01
    off = shard * d
    print("k5 shard", shard, dtype, flush=True)
    w, bias = _weights(Ci, Co, dtype, 530)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    xa = cut("uniform", SEED, 505, (N, Ci, Dg, H, W), off, d, (2, 2))
    xo, xg = slab_pair(xa, dtype, (2, 2), off, Dg)
    zo = orc.convk_fwd(xo, w, bias, orc.ACT_LEAKY, alpha)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    zg = h3d.Slab(torch.full((N, Co, d + 3, H, W), 12345.0, device="cuda", dtype=td), 1, 2, off, Dg)
    h3d.conv3d_k5_fwd(xg, wd, bd, zg, h3d.ACT_LEAKY, alpha)
    got = from_dev(zg.t)
    close(got[:, :, 1:-2], zo.a, TOL[dtype])
    canary = got[0, 0, 0, 0, 0]
    assert canary == 12345.0 or dtype == "bf16"
    assert np.all(got[:, :, 0] == canary) and np.all(got[:, :, -2:] == canary)
    # backward: dz and the saved z with two halo planes, cut from seeded full tensors
    full_z = (N, Co, Dg, H, W)
    dzo, dzg = slab_pair(cut("uniform", SEED, 506, full_z, off, d, (2, 2)), dtype, (2, 2), off, Dg)
    zso, zsg = slab_pair(cut("normal", SEED, 507, full_z, off, d, (2, 2)), dtype, (2, 2), off, Dg)
    dxo = orc.convk_bwd_data(dzo, zso, w, orc.ACT_LEAKY, alpha)
    dxg = h3d.conv3d_k5_bwd_data(dzg, zsg, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.convk_bwd_filter(5, xo, dzo, zso, orc.ACT_LEAKY, alpha)
    dw = torch.full((Co, Ci, 5, 5, 5), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_k5_bwd_filter(xg, dzg, zsg, dw, db, h3d.ACT_LEAKY, alpha)
    close(from_dev(dw), dwo, _tol_w(dtype))
    close(from_dev(db), dbo, _tol_w(dtype))


def test_k5_larger_volume_sampled_against_the_oracle_definition():
    """1 x 16 x 32^3 -> 32 channels in bf16: too slow for the whole oracle pass in a test; sampled output voxels are
    computed one by one from the definition (fp64 sum over the padded window)."""
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D = 1, 16, 32, 32
    print("k5 sampled 32^3", flush=True)
    w, bias = _weights(Ci, Co, "bf16", 540)
    x = quantize(synth.flat("uniform", SEED, 508, (N, Ci, D, D, D)), "bf16")
    _, xg = slab_pair(x, "bf16")
    zg = h3d.conv3d_k5_fwd(xg, to_dev(w, "bf16"), to_dev(bias, "f32"), dev_like(orc.Slab(np.zeros((N, Co, D, D, D))), "bf16"),
                           h3d.ACT_NONE, 0.0)
    got = from_dev(zg.t)
    xp = np.zeros((Ci, D + 4, D + 4, D + 4))
    xp[:, 2:-2, 2:-2, 2:-2] = x[0]
    rng = np.random.default_rng(SEED + 509)
    pts = [(0, 0, 0, 0), (Co - 1, D - 1, D - 1, D - 1), (5, 0, D - 1, 17), (17, 31, 0, 1)]
    pts += [tuple(int(v) for v in (rng.integers(Co), rng.integers(D), rng.integers(D), rng.integers(D))) for _ in range(200)]
    ref = np.array([bias[co] + np.sum(w[co] * xp[:, p:p + 5, h:h + 5, v:v + 5]) for co, p, h, v in pts])
    val = np.array([got[0, co, p, h, v] for co, p, h, v in pts])
    close(val, ref, TOL["bf16"])


def test_k5_backward_at_the_bench_shape_sampled_against_the_definition():
    """The launch configuration bench.py times (32 -> 32 channels, 128 x 128 planes, an interior shard with two halo
    planes per side, leaky-ReLU mask), on 8 interior planes: sampled dx voxels and dw entries are computed one by one
    from the definition in fp64 (g = dz * act'(z) taken from the unrounded product, as the oracle does)."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W, off, Dg, alpha = 1, 32, 8, 128, 128, 32, 128, 0.01
    print("k5 sampled backward at the bench shape", flush=True)
    w, _ = _weights(C, C, "bf16", 550)
    full = (N, C, Dg, H, W)
    xa = quantize(cut("uniform", SEED, 551, full, off, d, (2, 2)), "bf16")
    dza = quantize(cut("uniform", SEED, 552, full, off, d, (2, 2)), "bf16")
    za = quantize(cut("normal", SEED, 553, full, off, d, (2, 2)), "bf16")
    _, xg = slab_pair(xa, "bf16", (2, 2), off, Dg)
    _, dzg = slab_pair(dza, "bf16", (2, 2), off, Dg)
    _, zg = slab_pair(za, "bf16", (2, 2), off, Dg)
    g = dza * np.where(za > 0, 1.0, alpha)                       # [1, C, d+4, H, W], stored planes -2 .. d+1
    gp = np.zeros((C, d + 4, H + 4, W + 4)); gp[:, :, 2:-2, 2:-2] = g[0]
    xp = np.zeros((C, d + 4, H + 4, W + 4)); xp[:, :, 2:-2, 2:-2] = xa[0]
    rng = np.random.default_rng(SEED + 554)
    # backward-data: dx[ci,q,h,v] = sum_{co,k} w[co,ci,k] g~[co,q-k+2]  (window of g reversed against the filter)
    dxg = h3d.conv3d_k5_bwd_data(dzg, zg, to_dev(w, "bf16"), h3d.Slab(torch.full((N, C, d, H, W), 7.0, device="cuda", dtype=torch.bfloat16),
                                                                   0, 0, off, Dg), h3d.ACT_LEAKY, alpha)
    got = from_dev(dxg.t)
    pts = [(0, 0, 0, 0), (C - 1, d - 1, H - 1, W - 1), (3, 0, H - 1, 17), (17, d - 1, 0, 1)]
    pts += [tuple(int(v) for v in (rng.integers(C), rng.integers(d), rng.integers(H), rng.integers(W))) for _ in range(150)]
    ref = np.array([np.sum(w[:, ci, ::-1, ::-1, ::-1] * gp[:, q:q + 5, h:h + 5, v:v + 5]) for ci, q, h, v in pts])
    val = np.array([got[0, ci, q, h, v] for ci, q, h, v in pts])
    close(val, ref, TOL["bf16"])
    # backward-filter: dw[co,ci,k] = sum over the interior of g[co,p] x~[ci,p+k-2]; db[co] = sum g
    dw = torch.full((C, C, 5, 5, 5), 777.0, device="cuda")
    db = torch.full((C,), 777.0, device="cuda")
    h3d.conv3d_k5_bwd_filter(xg, dzg, zg, dw, db, h3d.ACT_LEAKY, alpha)
    gi = g[0][:, 2:-2]                                            # interior planes
    ent = [(0, 0, 0, 0, 0), (C - 1, C - 1, 4, 4, 4), (5, 9, 2, 2, 2), (31, 0, 0, 4, 1)]
    ent += [tuple(int(v) for v in (rng.integers(C), rng.integers(C), rng.integers(5), rng.integers(5), rng.integers(5))) for _ in range(60)]
    ref = np.array([np.sum(gi[co] * xp[ci, kd:kd + d, kh:kh + H, kw:kw + W]) for co, ci, kd, kh, kw in ent])
    gw = from_dev(dw)
    val = np.array([gw[e] for e in ent])
    close(val, ref, _tol_w("bf16"))
    close(from_dev(db), gi.sum(axis=(1, 2, 3)), _tol_w("bf16"))


def test_k5_errors_do_not_launch():
    import ctypes
    import torch
    import paper_2007_12856_amd as h3d
    w = torch.zeros((3, 2, 5, 5, 5), device="cuda")
    x1 = h3d.Slab(torch.zeros((1, 2, 4 + 1 + 2, 4, 4), device="cuda"), 1, 2, 4, 16)     # one lower halo plane only
    z = h3d.Slab(torch.zeros((1, 3, 4, 4, 4), device="cuda"), 0, 0, 4, 16)
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_k5_fwd(x1, w, None, z)
    assert e.value.status == -4
    dx = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda"), 0, 0, 4, 16)
    with pytest.raises(h3d.H3DError) as e:                                              # dz without halo planes
        h3d.conv3d_k5_bwd_data(z, None, w, dx)
    assert e.value.status == -4
    xs = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda"))
    with pytest.raises(h3d.H3DError) as e:                                              # extents differ
        h3d.conv3d_k5_fwd(xs, w, None, h3d.Slab(torch.zeros((1, 3, 4, 4, 5), device="cuda")))
    assert e.value.status == -1
    zs = h3d.Slab(torch.zeros((1, 3, 4, 4, 4), device="cuda"))
    st = h3d.lib().h3d_conv3d_k5_fwd(h3d.handle(), ctypes.byref(xs.desc()), ctypes.c_void_p(w.data_ptr()), None,
                                     ctypes.byref(zs.desc()), 0, 0.0, None, 0, None)
    assert st == -3
    # a shard next to the boundary needs only the planes that exist: one plane below the interior here
    xb = h3d.Slab(torch.zeros((1, 2, 1 + 4 + 2, 4, 4), device="cuda"), 1, 2, 1, 16)
    h3d.conv3d_k5_fwd(xb, w, None, h3d.Slab(torch.zeros((1, 3, 4, 4, 4), device="cuda"), 0, 0, 1, 16))


def test_k5_empty_shard():
    import torch
    import paper_2007_12856_amd as h3d
    x = h3d.Slab(torch.zeros((1, 2, 0, 4, 4), device="cuda"), 0, 0, 0, 8)
    z = h3d.Slab(torch.zeros((1, 3, 0, 4, 4), device="cuda"), 0, 0, 0, 8)
    w = torch.zeros((3, 2, 5, 5, 5), device="cuda")
    h3d.conv3d_k5_fwd(x, w, None, z)
    dw = torch.full((3, 2, 5, 5, 5), 5.0, device="cuda")
    db = torch.full((3,), 5.0, device="cuda")
    h3d.conv3d_k5_bwd_filter(x, z, None, dw, db)
    torch.cuda.synchronize()
    assert float(dw.abs().max()) == 0.0 and float(db.abs().max()) == 0.0
