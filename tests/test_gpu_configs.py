"""Parity at the FULL sizes of the five benchmark configurations, in the launch configuration the
bench uses (relative L2 over each tensor and an element-by-element bound, helpers.close).  Where the full oracle would take minutes, the oracle computes SAMPLED outputs exactly
(whole output depth planes through 1-plane sub-slabs cut at the same global offsets, and channel
subsets through sliced weight tensors) while the GPU kernel runs the full shape.  Planes the
sampled outputs do not depend on hold seeded torch noise on the GPU only.
"""
import numpy as np
import pytest

import oracle as orc
import synth
from synth import recipes
from helpers import TOL, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED + 77
BF = "bf16"


def _tdt(dtype):
    import torch
    return torch.float32 if dtype == "f32" else torch.bfloat16


def _noise(shape, seed, dtype=BF):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(_tdt(dtype))


def _planes(kind, stream, full_shape, g_lo, g_hi, dtype=BF):
    """storage-rounded float64 global planes [g_lo, g_hi) of the seeded virtual tensor (zero outside the volume)."""
    return quantize(synth.slab(kind, SEED, stream, full_shape, g_lo, g_hi), dtype)


def _put(t, stored_lo, a, dtype=BF):
    """upload planes `a` into stored planes [stored_lo, ...) of device tensor t, clipped to what is stored"""
    lo, hi = max(stored_lo, 0), min(stored_lo + a.shape[2], t.shape[2])
    if hi > lo:
        t[:, :, lo:hi] = to_dev(a[:, :, lo - stored_lo:hi - stored_lo], dtype)


def sampled_conv_case(cin, cout, n, d, hw, halo_in, halo_out, d_offset, d_global, planes, nsub=8, kinds=("cosmo", "normal"),
                      act=orc.ACT_LEAKY, alpha=0.01, stream=0, dtype=BF):
    """fwd / bwd-data / bwd-filter of one conv layer at full shape against sampled oracle outputs."""
    import torch
    import paper_2007_12856_amd as h3d
    H = W = hw
    b = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, stream + 1, (cout, cin, 3, 3, 3), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, stream + 2, (cout,), -0.1, 0.1)).astype(np.float64)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    tdt, tol_w = _tdt(dtype), (1e-5 if dtype == "f32" else 2e-4)
    cos = np.unique(np.linspace(0, cout - 1, min(nsub, cout)).astype(int))
    cis = np.unique(np.linspace(0, cin - 1, min(nsub, cin)).astype(int))
    xfull, zfull = (n, cin, d_global, H, W), (n, cout, d_global, H, W)

    # ---------------- forward
    x = h3d.Slab(_noise((n, cin, d + 2 * halo_in, H, W), 1, dtype), halo_in, halo_in, d_offset, d_global)
    subs = {}
    for p in planes:      # local output plane index (may be a halo plane of z)
        a = _planes(kinds[0], stream + 3, xfull, d_offset + p - 1, d_offset + p + 2, dtype)
        _put(x.t, p - 1 + halo_in, a, dtype)
        subs[p] = orc.Slab(a, 1, 1, d_offset + p, d_global) if 0 <= d_offset + p < d_global else None
    z = h3d.Slab(torch.empty((n, cout, d + 2 * halo_out, H, W), dtype=tdt, device="cuda"), halo_out, halo_out,
                 d_offset, d_global)
    h3d.conv3d_fwd(x, wd, bd, z, act, alpha)
    for p in planes:
        got = from_dev(z.t[:, cos, p + halo_out])
        if subs[p] is None:
            assert not got.any()          # beyond the global boundary: zero padding of the next layer
            continue
        ref = orc.conv3d_fwd(subs[p], w[cos], bias[cos], act=act, alpha=alpha).a[:, :, 0]
        close(got, ref, TOL[dtype], f"fwd plane {p}")

    # ---------------- backward-data (dz and the saved output z carry a 1-plane exchanged halo)
    ip = [p for p in planes if 0 <= p < d]
    dz = h3d.Slab(_noise((n, cout, d + 2, H, W), 2, dtype), 1, 1, d_offset, d_global)
    zs = h3d.Slab(_noise((n, cout, d + 2, H, W), 3, dtype), 1, 1, d_offset, d_global)
    dzp, zp = {}, {}
    for p in ip:
        dzp[p] = _planes(kinds[1], stream + 4, zfull, d_offset + p - 1, d_offset + p + 2, dtype)
        zp[p] = _planes("normal", stream + 5, zfull, d_offset + p - 1, d_offset + p + 2, dtype)
        _put(dz.t, p, dzp[p], dtype)
        _put(zs.t, p, zp[p], dtype)
    dx = h3d.Slab(torch.empty((n, cin, d, H, W), dtype=tdt, device="cuda"), 0, 0, d_offset, d_global)
    h3d.conv3d_bwd_data(dz, zs, wd, dx, act, alpha)
    for p in ip:
        ref = orc.conv3d_bwd_data(orc.Slab(dzp[p], 1, 1, d_offset + p, d_global), orc.Slab(zp[p], 1, 1, d_offset + p, d_global),
                                  w[:, cis], act=act, alpha=alpha).a[:, :, 0]
        close(from_dev(dx.t[:, cis, p]), ref, TOL[dtype], f"bwd_data plane {p}")

    # ---------------- backward-filter: dz is zero outside the sampled planes on both sides
    dz0 = h3d.Slab(torch.zeros((n, cout, d, H, W), dtype=tdt, device="cuda"), 0, 0, d_offset, d_global)
    z0 = h3d.Slab(zs.t[:, :, 1:-1].contiguous(), 0, 0, d_offset, d_global)
    dw_ref, db_ref = 0.0, 0.0
    for p in ip:
        _put(dz0.t, p, dzp[p][:, :, 1:2], dtype)
        xa = _planes(kinds[0], stream + 3, xfull, d_offset + p - 1, d_offset + p + 2, dtype)
        _put(x.t, p - 1 + halo_in, xa, dtype)
        a, bq = orc.conv3d_bwd_filter(orc.Slab(xa[:, cis], 1, 1, d_offset + p, d_global),
                                      orc.Slab(dzp[p][:, cos, 1:2], 0, 0, d_offset + p, d_global),
                                      orc.Slab(zp[p][:, cos, 1:2], 0, 0, d_offset + p, d_global), act=act, alpha=alpha)
        dw_ref, db_ref = dw_ref + a, db_ref + bq
    dw = torch.empty((cout, cin, 3, 3, 3), device="cuda")
    db = torch.empty((cout,), device="cuda")
    h3d.conv3d_bwd_filter(x, dz0, z0, dw, db, act, alpha)
    got = from_dev(dw)[cos][:, cis]
    close(got, dw_ref, tol_w, "bwd_filter dw")
    close(from_dev(db)[cos], db_ref, tol_w, "bwd_filter db")
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_bwd_filter(x, dz0, z0, dw2, db2, act, alpha)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)      # deterministic split-spatial reduction
    # the same call without a fused mask (the activation's derivative already applied upstream, as the benchmark's
    # steps do it): at full shape this is the route to the unmasked kernels and their many-strip chunks
    dwu_ref, dbu_ref = 0.0, 0.0
    for p in ip:
        xa = _planes(kinds[0], stream + 3, xfull, d_offset + p - 1, d_offset + p + 2, dtype)
        a, bq = orc.conv3d_bwd_filter(orc.Slab(xa[:, cis], 1, 1, d_offset + p, d_global),
                                      orc.Slab(dzp[p][:, cos, 1:2], 0, 0, d_offset + p, d_global), None, act=orc.ACT_NONE)
        dwu_ref, dbu_ref = dwu_ref + a, dbu_ref + bq
    h3d.conv3d_bwd_filter(x, dz0, None, dw, db, h3d.ACT_NONE, 0.0)
    close(from_dev(dw)[cos][:, cis], dwu_ref, tol_w, "unmasked bwd_filter dw")
    close(from_dev(db)[cos], dbu_ref, tol_w, "unmasked bwd_filter db")
    h3d.conv3d_bwd_filter(x, dz0, None, dw2, db2, h3d.ACT_NONE, 0.0)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)
    return z


# ---------------------------------------------------------------- configuration 1
def test_cfg1_single_layer_fp32():
    """N=1, 4->16, 32^3, fp32, bias + leaky-ReLU 0.01, inputs/weights/gradient uniform in [-1,1]; full oracle."""
    import torch
    import paper_2007_12856_amd as h3d
    f = "f32"
    w = quantize(synth.flat("uniform", SEED, 1, (16, 4, 3, 3, 3)), f)
    bias = quantize(synth.flat("uniform", SEED, 2, (16,), -0.1, 0.1), f)
    xo, xg = slab_pair(synth.flat("uniform", SEED, 3, (1, 4, 32, 32, 32)), f)
    dzo, dzg = slab_pair(synth.flat("uniform", SEED, 4, (1, 16, 32, 32, 32)), f)
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=0.01)
    zg = h3d.conv3d_fwd(xg, to_dev(w, f), to_dev(bias, f), dev_like(zo, f), h3d.ACT_LEAKY, 0.01)
    close(from_dev(zg.t), zo.a, 1e-5)
    zqo, zqg = slab_pair(zo.a, f)
    dxo = orc.conv3d_bwd_data(dzo, zqo, w, act=orc.ACT_LEAKY, alpha=0.01)
    dxg = h3d.conv3d_bwd_data(dzg, zqg, to_dev(w, f), dev_like(dxo, f), h3d.ACT_LEAKY, 0.01)
    close(from_dev(dxg.t), dxo.a, 1e-5)
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, zqo, act=orc.ACT_LEAKY, alpha=0.01)
    dw, db = torch.empty((16, 4, 3, 3, 3), device="cuda"), torch.empty((16,), device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, zqg, dw, db, h3d.ACT_LEAKY, 0.01)
    close(from_dev(dw), dwo, 1e-5)
    close(from_dev(db), dbo, 1e-5)


# ---------------------------------------------------------------- configuration 2
def test_cfg2_cosmoflow_stack_full_size():
    """N=4 x 4x128^3 bf16, five conv+leaky+avg-pool stages, dense 16384-2048-256-4, MSE, fwd+bwd, built and run exactly
    as bench.py times it: first stage fused (conv + pooling forward, sign mask, no stored activation), pooling backward
    from a sign mask, the backward-filter calls of the late stages and the dense weight gradients on a second stream.
    Two comparisons, both on the whole batch (FP, BD and BF of every layer, Sec. III-C, on the shapes of Table I's first stages):
    A. the step against the oracle's evaluation of the same network on the same bf16 inputs and weights (fp64 sums, stored
       tensors rounded to bf16 as on the GPU), every tensor on the bf16 bar: forward, loss and loss gradient in one
       unbroken pass; the backward pass of the convolution stages from the oracle's gradient at the flatten;
    B. every backward stage (dense head, then each convolution stage) once more from IDENTICAL inputs (the oracle's
       tensors, rounded to bf16, uploaded into the stage's buffers), on the bars of the single calls: bf16 results one
       rounding, fp32 filter gradients 2e-4."""
    import torch
    from test_gpu_stack import BWD_ELEM, FWD_ELEM, build, loss_bound
    from oracle_nets import cosmoflow_oracle
    net, xq, tq, convq, fcq = build(BF, 4, 128, recipes.COSMO_CHANNELS, recipes.COSMO_FC, synth.BASE_SEED, fuse_pool=True)
    net.overlap = True
    # (the last stage's 8-voxel rows are too short for the mask kernels: its pooling backward reads the stored activation)
    assert net.fused == [True, False, False, False, False] and [m is not None for m in net.mask] == [True, True, True, True, False]
    names = [o["name"] for o in net.ops]
    assert names[:3] == ["conv1_fwd_pool", "conv2_fwd", "pool2_fwd"]
    assert "pool1_bwd_mask" in names and "pool4_bwd_mask" in names and "pool5_bwd_act" in names
    net.step()
    torch.cuda.synchronize()
    assert net.side is not None                         # the second stream was used
    tol, alpha = TOL[BF], 0.01
    qz = lambda v: quantize(v, BF)
    # The oracle rounds every STORED tensor to bf16 as the GPU does (sums in fp64).  Against the network evaluated without
    # that rounding the forward tensors agree to 2-3e-3, but the backward pass cannot be compared: the slope of a leaky
    # ReLU is taken from the sign of the stored activation, a relative difference of 2.5e-3 between the two forward
    # passes puts about 0.2 % of the activations on different sides of zero, and a fraction f of voxels with the slope
    # off by a factor of 100 is a relative L2 difference of sqrt(2 f) = 6e-2 in g (measured: 3.6e-2 after one stage,
    # 7e-2 after five).  With the storage format part of each layer's contract on both sides the forward passes differ
    # by 1e-5 .. 1e-3 and such flips are rare.
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=qz)
    # ---- A: the unbroken step
    close(from_dev(net.p[0].t), ref["p"][0].a, tol, "p1", **FWD_ELEM[BF])
    for i in range(1, 5):
        close(from_dev(net.z[i].t), ref["z"][i].a, tol, f"z{i + 1}", **FWD_ELEM[BF])
        close(from_dev(net.p[i].t), ref["p"][i].a, tol, f"p{i + 1}", **FWD_ELEM[BF])
    # the mask the fused first stage wrote: the oracle's, except where the activation is within rounding of zero
    want = orc.act_mask(ref["z"][0])
    got = net.mask[0].cpu().numpy().reshape(want.shape)
    diff = np.unpackbits((got ^ want)[..., None], axis=-1, bitorder="little").reshape(ref["z"][0].a.shape).astype(bool)
    assert diff.mean() < 1e-3 and np.all(np.abs(ref["z"][0].a[diff]) <= 1e-2 * np.abs(ref["z"][0].a).max())
    del want, got, diff
    pred = ref["y"][-1]
    close(from_dev(net.y[-1]), pred, tol, "pred")
    assert abs(net.loss.item() - ref["loss"]) <= loss_bound(pred, tq, tol) * abs(ref["loss"])
    # the loss gradient turns a relative difference e of pred into e |pred| / |pred - t| of itself (the MSE call is
    # compared on identical inputs in test_dense_and_mse); with targets in [-1, 1] and small predictions that factor is < 1
    amp = np.linalg.norm(pred) / np.linalg.norm(pred - tq)
    close(from_dev(net.dy[-1]), ref["dpred"], tol * max(1.0, amp), "loss gradient")
    # The backward pass of the convolution stages, as the step runs it, from the oracle's gradient at the flatten.  (The
    # dense head is cut off here and compared from identical inputs below: its layers have 256 and 2048 outputs per
    # sample, and ONE activation within rounding of zero whose sign differs between the two forward passes changes the
    # slope of that output from 0.01 to 1 - a few per cent of such a small layer's gradient norm, passed on unchanged to
    # every tensor below.  In the convolution stages the same flips are a vanishing share of millions of voxels.)
    net.dp[4].t.copy_(to_dev(qz(ref["dp"][4].a), BF))
    ops = {o["name"]: o["fn"] for o in net.ops}
    for o in net.ops[names.index("pool5_bwd_act"):]:
        o["fn"]()
    torch.cuda.synchronize()
    # element by element here only coarsely: stage 5's activations differ by 1.2e-3 between the two forward passes, 1e-4 of
    # them lie on different sides of zero, which alone is sqrt(2e-4) = 1.4e-2 of g5's norm and is spread by every
    # backward-data convolution below; part B holds every element of every stage to the single-call bounds
    coarse = dict(elem=2.0 ** -3, outliers=2e-3)
    for i in range(5):
        close(from_dev(net.g[i].t), ref["g"][i].a, tol, f"g{i + 1}", **coarse)
        close(from_dev(net.dconv[i][0]), ref["dconv"][i][0], tol, f"dw{i + 1}", **coarse)
        close(from_dev(net.dconv[i][1]), ref["dconv"][i][1], tol, f"db{i + 1}", **coarse)
    close(from_dev(net.dx.t), ref["dx"].a, tol, "dx", **coarse)
    # the two-stream schedule is deterministic: the whole backward pass twice, identical bits
    net.backward()
    torch.cuda.synchronize()
    grads = lambda: [t for pair in net.dconv + net.dfc for t in pair] + [net.dx.t]
    keep = [t.clone() for t in grads()]
    for t in grads():
        t.fill_(3.0)
    net.backward()
    torch.cuda.synchronize()
    for a, b in zip(keep, grads()):
        assert torch.equal(a, b)
    del keep
    # ---- B: the dense head's backward from identical inputs (BD and BF of the fully-connected layers)
    hq = [qz(ref["p"][4].a).reshape(4, -1)] + [qz(y) for y in ref["y"]]
    net.p[4].t.copy_(to_dev(hq[0].reshape(ref["p"][4].a.shape), BF))
    for i in range(3):
        net.y[i].copy_(to_dev(hq[i + 1], BF))
    g = qz(ref["dpred"])
    for i in (2, 1, 0):
        net.dy[i].copy_(to_dev(g, BF))
        ops[f"fc{i + 1}_bwd"]()
        ops["join"]()
        torch.cuda.synchronize()
        g, dw, db = orc.dense_bwd(hq[i], fcq[i][0], hq[i + 1], g, orc.ACT_NONE if i == 2 else orc.ACT_LEAKY, alpha)
        close(from_dev(net.dfc[i][0]), dw, tol, f"fc{i + 1} dw")
        close(from_dev(net.dfc[i][1]), db, tol, f"fc{i + 1} db")
        close(from_dev(net.dp[4].t).reshape(4, -1) if i == 0 else from_dev(net.dy[i - 1]), g, tol, f"fc{i + 1} dx")
        g = qz(g)
    # ---- B: the convolution stages one by one from identical inputs, with the calls (and streams) of the step
    for i in range(4, -1, -1):
        w = convq[i][0]
        zq = orc.Slab(qz(ref["z"][i].a))
        dpq = orc.Slab(qz(ref["dp"][i].a))
        xin = orc.Slab(xq) if i == 0 else orc.Slab(qz(ref["out"][i - 1].a))
        net.dp[i].t.copy_(to_dev(dpq.a, BF))
        if i > 0:
            net.out[i - 1].t.copy_(to_dev(xin.a, BF))
        if net.z[i] is not None:
            net.z[i].t.copy_(to_dev(zq.a, BF))
        if net.mask[i] is not None:
            net.mask[i].copy_(torch.from_numpy(orc.act_mask(zq).ravel()).cuda())
        for nm in (f"pool{i + 1}_bwd_mask", f"pool{i + 1}_bwd_act"):
            if nm in ops:
                ops[nm]()
        ops[f"conv{i + 1}_bwd_filter"]()
        ops[f"conv{i + 1}_bwd_data"]()
        ops["join"]()
        torch.cuda.synchronize()
        g = orc.act_bwd(orc.pool3d_bwd(dpq, None, orc.POOL_AVG), None, zq, orc.ACT_LEAKY, alpha)
        close(from_dev(net.g[i].t), g.a, 4e-3, f"stage {i + 1} g", elem=2.0 ** -8)       # one bf16 rounding of an exact product
        gq = orc.Slab(qz(g.a))
        dw, db = orc.conv3d_bwd_filter(xin, gq, None)
        close(from_dev(net.dconv[i][0]), dw, 2e-4, f"stage {i + 1} dw")
        close(from_dev(net.dconv[i][1]), db, 2e-4, f"stage {i + 1} db")
        dxi = orc.conv3d_bwd_data(gq, None, w)
        close(from_dev((net.dx if i == 0 else net.dout[i - 1]).t), dxi.a, tol, f"stage {i + 1} dx")
        del g, gq, dw, db, dxi, zq, dpq, xin


def test_fp32_layer_of_the_bench_full_size():
    """The fp32 layer that `bench.py --workload layer_f32` times (32->64 channels on a whole 32x128x128 volume): the fp32
    matrix-core kernels at their 8-row, two-half tiles, against sampled oracle planes at the fp32 bar."""
    sampled_conv_case(32, 64, 1, 32, 128, 1, 0, 0, 32, [0, 15, 31], kinds=("normal", "normal"), stream=400, dtype="f32")


# ---------------------------------------------------------------- configuration 3
@pytest.mark.parametrize("d_offset,planes", [(64, [0, 31, 63]), (0, [0]), (448, [63])])
def test_cfg3_shard_of_512cube_first_layer(d_offset, planes):
    """One 8-way depth shard of a 4-channel 512^3 sample: 4x66x512x512 bf16, conv 4->16 + leaky."""
    sampled_conv_case(4, 16, 1, 64, 512, 1, 0, d_offset, 512, planes, stream=100)


def test_cfg3_pool_and_halo_at_full_size():
    import torch
    import paper_2007_12856_amd as h3d
    z = h3d.Slab(_noise((1, 16, 66, 512, 512), 5), 1, 1, 64, 512)
    p = h3d.Slab(torch.empty((1, 16, 32, 256, 256), dtype=torch.bfloat16, device="cuda"), 0, 0, 32, 256)
    h3d.pool3d_fwd(z, p, h3d.POOL_AVG)
    dp = h3d.Slab(_noise((1, 16, 32, 256, 256), 6), 0, 0, 32, 256)
    dz = h3d.Slab(torch.empty((1, 16, 64, 512, 512), dtype=torch.bfloat16, device="cuda"), 0, 0, 64, 512)
    h3d.pool3d_bwd(dp, None, dz, h3d.POOL_AVG)
    for q in (0, 17, 31):      # pooled plane q <- planes 2q, 2q+1 of the interior
        zin = orc.Slab(from_dev(z.t[:, :, 1 + 2 * q:3 + 2 * q]), 0, 0, 64 + 2 * q, 512)
        close(from_dev(p.t[:, :, q]), orc.pool3d_fwd(zin, orc.POOL_AVG).a[:, :, 0], 4e-3)
        ref = orc.pool3d_bwd(orc.Slab(from_dev(dp.t[:, :, q:q + 1])), None, orc.POOL_AVG).a
        close(from_dev(dz.t[:, :, 2 * q:2 * q + 2]), ref, 4e-3)
    # halo pack/unpack of both D faces: input faces (4 ch) and activation faces (16 ch), bit-exact
    for t in (h3d.Slab(_noise((1, 4, 66, 512, 512), 7), 1, 1, 64, 512), z):
        o = orc.Slab(from_dev(t.t), 1, 1, 64, 512)
        for face in (h3d.FACE_D_LO, h3d.FACE_D_HI):
            buf = torch.empty(h3d.halo_bytes(t, 1) // 2, dtype=torch.bfloat16, device="cuda")
            h3d.halo_pack(t, face, 1, buf)
            assert np.array_equal(from_dev(buf).reshape(orc.halo_pack(o, face, 1).shape), orc.halo_pack(o, face, 1))
            h3d.halo_unpack(buf, t, 1 - face, 1)
            orc.halo_unpack(orc.halo_pack(o, face, 1), o, 1 - face, 1)
        assert np.array_equal(from_dev(t.t), o.a)


def test_cfg3_fused_first_layer_full_size():
    """The first layer of the shard as `bench.py --workload shard512` runs it: convolution + leaky-ReLU + 2x2x2 average
    pooling in ONE call that stores no unpooled activation but its sign mask, and the pooling backward that reads the mask.
    Sampled pooled planes against the oracle's composition conv -> store as bf16 -> pool (Sec. III-C FP; Table I shapes)."""
    import torch
    import paper_2007_12856_amd as h3d
    n, cin, cout, d, hw, off, dg, alpha = 1, 4, 16, 64, 512, 64, 512, 0.01
    bnd = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, 111, (cout, cin, 3, 3, 3), -bnd, bnd), BF)
    bias = synth.round_f32(synth.flat("uniform", SEED, 112, (cout,), -0.1, 0.1)).astype(np.float64)
    x = h3d.Slab(_noise((n, cin, d + 2, hw, hw), 21), 1, 1, off, dg)
    qs, xs = (0, 17, 31), {}
    for q in qs:                                   # pooled plane q <- output planes 2q, 2q+1 <- input planes 2q-1 .. 2q+2
        xs[q] = _planes("cosmo", 113, (n, cin, dg, hw, hw), off + 2 * q - 1, off + 2 * q + 3)
        _put(x.t, 2 * q, xs[q])
    y = h3d.Slab(torch.empty((n, cout, d // 2, hw // 2, hw // 2), dtype=torch.bfloat16, device="cuda"), 0, 0, off // 2, dg // 2)
    mask = torch.full((n * cout * d * hw * hw // 8,), 0xAA, dtype=torch.uint8, device="cuda")
    h3d.conv3d_fwd_pool(x, to_dev(w, BF), to_dev(bias, "f32"), (n, cout, d, hw, hw), y, mask, h3d.ACT_LEAKY, alpha)
    assert h3d.h3d_last_kernel().startswith("conv3d_fwd_c4_roll"), h3d.h3d_last_kernel()
    mk = mask.cpu().numpy().reshape(n, cout, d, hw, hw // 8)
    for q in qs:
        zo = orc.conv3d_fwd(orc.Slab(xs[q], 1, 1, off + 2 * q, dg), w, bias, act=orc.ACT_LEAKY, alpha=alpha)
        zq = orc.Slab(quantize(zo.a, BF), 0, 0, off + 2 * q, dg)
        close(from_dev(y.t[:, :, q]), orc.pool3d_fwd(zq, orc.POOL_AVG).a[:, :, 0], 4e-3, f"pooled plane {q}")
        # the mask is the sign of the activation; the two sides may differ where it is within rounding of zero
        diff = np.unpackbits((mk[:, :, 2 * q:2 * q + 2] ^ orc.act_mask(zq))[..., None], axis=-1, bitorder="little")
        diff = diff.reshape(zo.a.shape).astype(bool)
        assert np.all(np.abs(zo.a[diff]) <= 1e-2 * np.abs(zo.a).max()) and diff.mean() < 1e-3, f"mask of planes {2 * q}, {2 * q + 1}"
    # pooling backward from the mask: g = pool'(dp) * act'(z), the sign taken from the stored mask on both sides
    dp = h3d.Slab(_noise((n, cout, d // 2, hw // 2, hw // 2), 22), 0, 0, off // 2, dg // 2)
    g = h3d.Slab(torch.full((n, cout, d + 2, hw, hw), 7.0, dtype=torch.bfloat16, device="cuda"), 1, 1, off, dg)
    h3d.pool3d_bwd_mask(dp, mask, g, h3d.ACT_LEAKY, alpha)
    for q in qs:
        up = orc.pool3d_bwd(orc.Slab(from_dev(dp.t[:, :, q:q + 1])), None, orc.POOL_AVG).a
        pos = np.unpackbits(mk[:, :, 2 * q:2 * q + 2][..., None], axis=-1, bitorder="little").reshape(up.shape).astype(bool)
        close(from_dev(g.t[:, :, 1 + 2 * q:3 + 2 * q]), up * np.where(pos, 1.0, alpha), 4e-3, f"g planes {2 * q}, {2 * q + 1}")
    assert torch.all(g.t[:, :, 0] == 7.0) and torch.all(g.t[:, :, -1] == 7.0)        # halo planes are the neighbours': untouched


# ---------------------------------------------------------------- configuration 4 (layers at full shape)
@pytest.mark.parametrize("name,cin,cout,d,hw,halo_in,halo_out,dg,planes", [
    ("c1", 1, 32, 64, 256, 2, 1, 256, [-1, 30, 64]),
    ("c2", 32, 64, 64, 256, 1, 0, 256, [0, 63]),
    ("c3", 64, 64, 32, 128, 2, 1, 128, [-1, 31]),
    ("c4", 64, 128, 32, 128, 1, 0, 128, [0, 17]),
    ("c6", 128, 64, 64, 256, 1, 0, 256, [5, 63]),
])
def test_cfg4_unet_layers_full_size(name, cin, cout, d, hw, halo_in, halo_out, dg, planes):
    sampled_conv_case(cin, cout, 1, d, hw, halo_in, halo_out, d * 1, dg, planes, kinds=("normal", "normal"),
                      act=orc.ACT_RELU, alpha=0.0, stream=200 + 10 * len(name) + cin)


def test_cfg4_first_shard_halo_plane_is_zero():
    """Boundary shard (d_offset 0) of the 1->32 layer with halo recompute: the output plane beyond the
    volume must be zero, not act(bias)."""
    sampled_conv_case(1, 32, 1, 64, 256, 2, 1, 0, 256, [-1, 0], kinds=("normal", "normal"), act=orc.ACT_RELU, alpha=0.0, stream=290)


def test_cfg4_deconv_maxpool_concat_full_size():
    import torch
    import paper_2007_12856_amd as h3d
    # 2x2x2 stride-2 transposed conv 128 -> 64 from 32x128x128 up to 64x256x256; sampled coarse planes
    b = np.sqrt(3.0 / (8 * 128))
    w = quantize(synth.flat("uniform", SEED, 301, (128, 64, 2, 2, 2), -b, b), BF)
    bias = synth.round_f32(synth.flat("uniform", SEED, 302, (64,), -0.1, 0.1)).astype(np.float64)
    x = h3d.Slab(_noise((1, 128, 32, 128, 128), 11), 0, 0, 32, 128)
    y = h3d.Slab(torch.empty((1, 64, 64, 256, 256), dtype=torch.bfloat16, device="cuda"), 0, 0, 64, 256)
    cos = np.arange(0, 64, 8)
    planes = [0, 13, 31]
    xp = {q: _planes("normal", 303, (1, 128, 128, 128, 128), 32 + q, 33 + q) for q in planes}
    for q in planes:
        _put(x.t, q, xp[q])
    h3d.deconv2_fwd(x, to_dev(w, BF), to_dev(bias, "f32"), y)
    for q in planes:
        ref = orc.deconv2_fwd(orc.Slab(xp[q], 0, 0, 32 + q, 128), w[:, cos], bias[cos]).a
        close(from_dev(y.t[:, cos, 2 * q:2 * q + 2]), ref, TOL[BF])
    dy = h3d.Slab(_noise((1, 64, 64, 256, 256), 12), 0, 0, 64, 256)
    dyp = {q: _planes("normal", 304, (1, 64, 256, 256, 256), 64 + 2 * q, 66 + 2 * q) for q in planes}
    for q in planes:
        _put(dy.t, 2 * q, dyp[q])
    dx = h3d.Slab(torch.empty((1, 128, 32, 128, 128), dtype=torch.bfloat16, device="cuda"), 0, 0, 32, 128)
    h3d.deconv2_bwd_data(dy, to_dev(w, BF), dx)
    cis = np.arange(0, 128, 16)
    for q in planes:
        ref = orc.deconv2_bwd_data(orc.Slab(dyp[q], 0, 0, 64 + 2 * q, 256), w[cis]).a
        close(from_dev(dx.t[:, cis, q:q + 1]), ref, TOL[BF])
    dy0 = h3d.Slab(torch.zeros_like(dy.t), 0, 0, 64, 256)
    dwr, dbr = 0.0, 0.0
    for q in planes:
        _put(dy0.t, 2 * q, dyp[q])
        a, bb = orc.deconv2_bwd_filter(orc.Slab(xp[q][:, cis], 0, 0, 32 + q, 128), orc.Slab(dyp[q][:, cos], 0, 0, 64 + 2 * q, 256))
        dwr, dbr = dwr + a, dbr + bb
    dw, db = torch.empty((128, 64, 2, 2, 2), device="cuda"), torch.empty((64,), device="cuda")
    h3d.deconv2_bwd_filter(x, dy0, dw, db)
    close(from_dev(dw)[cis][:, cos], dwr, 2e-4)
    close(from_dev(db)[cos], dbr, 2e-4)
    # max-pool 64 ch 64x256x256 -> 32x128x128 (forward exact, routing exact incl. ties after ReLU)
    a2 = h3d.Slab(torch.relu(_noise((1, 64, 64, 256, 256), 13)), 0, 0, 64, 256)
    p = h3d.Slab(torch.empty((1, 64, 32, 128, 128), dtype=torch.bfloat16, device="cuda"), 0, 0, 32, 128)
    h3d.pool3d_fwd(a2, p, h3d.POOL_MAX)
    dpl = h3d.Slab(_noise((1, 64, 32, 128, 128), 14), 0, 0, 32, 128)
    da2 = h3d.Slab(torch.empty_like(a2.t), 0, 0, 64, 256)
    h3d.pool3d_bwd(dpl, a2, da2, h3d.POOL_MAX)
    for q in (0, 31):
        xin = orc.Slab(from_dev(a2.t[:, :, 2 * q:2 * q + 2]), 0, 0, 64 + 2 * q, 256)
        assert np.array_equal(from_dev(p.t[:, :, q]), orc.pool3d_fwd(xin, orc.POOL_MAX).a[:, :, 0])
        ref = orc.pool3d_bwd(orc.Slab(from_dev(dpl.t[:, :, q:q + 1])), xin, orc.POOL_MAX).a
        assert np.array_equal(from_dev(da2.t[:, :, 2 * q:2 * q + 2]), ref)
    # concat skip (64) + up (64) into a 128-channel slab with a 1-plane halo, then split back: bit-exact
    cat = h3d.Slab(torch.full((1, 128, 66, 256, 256), 3.0, dtype=torch.bfloat16, device="cuda"), 1, 1, 64, 256)
    h3d.concat_c(a2, y, cat)
    assert torch.equal(cat.t[:, :64, 1:-1], a2.t) and torch.equal(cat.t[:, 64:, 1:-1], y.t)
    assert bool((cat.t[:, :, [0, -1]] == 3.0).all())
    s1, s2 = h3d.Slab(torch.empty_like(a2.t), 0, 0, 64, 256), h3d.Slab(torch.empty_like(y.t), 0, 0, 64, 256)
    h3d.split_c(cat, s1, s2)
    assert torch.equal(s1.t, a2.t) and torch.equal(s2.t, y.t)


# ---------------------------------------------------------------- configuration 5
def test_cfg5_late_layer_256x256_channel_sampled():
    """N=8, 256->256, 16^3, bf16: weight-gradient-bound late layer.  The GPU runs the full shape; the
    oracle computes 8 of the 256 output (fwd, BF) / input (BD, BF) channels, two samples for fwd and BD,
    all eight samples for the weight gradient."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, S = 8, 256, 16
    b = np.sqrt(3.0 / 6912)
    w = quantize(synth.flat("uniform", SEED, 401, (C, C, 3, 3, 3), -b, b), BF)
    xq = quantize(synth.flat("normal", SEED, 402, (N, C, S, S, S)), BF)
    dzq = quantize(synth.flat("normal", SEED, 403, (N, C, S, S, S)), BF)
    sub = np.arange(5, 256, 32)
    ns = [0, 7]
    x, dz = h3d.Slab(to_dev(xq, BF)), h3d.Slab(to_dev(dzq, BF))
    z = h3d.Slab(torch.empty_like(x.t))
    h3d.conv3d_fwd(x, to_dev(w, BF), None, z)
    ref = orc.conv3d_fwd(orc.Slab(xq[ns]), w[sub], None).a
    close(from_dev(z.t[ns][:, sub]), ref, TOL[BF])
    dx = h3d.Slab(torch.empty_like(x.t))
    h3d.conv3d_bwd_data(dz, None, to_dev(w, BF), dx)
    ref = orc.conv3d_bwd_data(orc.Slab(dzq[ns]), None, w[:, sub]).a
    close(from_dev(dx.t[ns][:, sub]), ref, TOL[BF])
    dw, db = torch.empty((C, C, 3, 3, 3), device="cuda"), torch.empty((C,), device="cuda")
    h3d.conv3d_bwd_filter(x, dz, None, dw, db)
    dwr, dbr = orc.conv3d_bwd_filter(orc.Slab(xq[:, sub]), orc.Slab(dzq[:, sub]), None)
    close(from_dev(dw)[sub][:, sub], dwr, 2e-4)
    close(from_dev(db)[sub], dbr, 2e-4)
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_bwd_filter(x, dz, None, dw2, db2)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)
