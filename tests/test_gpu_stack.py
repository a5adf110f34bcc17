"""Whole-stack parity: the CosmoFlow-shaped network (conv+leaky+avg-pool stages, dense head, MSE),
forward and backward, HIP path vs the oracle on identical seeded bf16/fp32 inputs."""
import numpy as np
import pytest

import synth
from synth import recipes
from helpers import from_dev, quantize, rel_l2, to_dev
from oracle_nets import cosmoflow_oracle, shard_chain_oracle

pytestmark = pytest.mark.gpu


def build(dtype, n, width, channels, fc, seed, fuse_pool=False, strides=None, pools=None, flat_w=None, bias=True):
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import CosmoFlowStack
    P = recipes.cosmoflow_params(seed, width, channels, fc, flat_w)
    x, t = recipes.cosmoflow_batch(seed, n, width, channels[0], fc[-1])
    convq = [(quantize(w, dtype), synth.round_f32(b).astype(np.float64) if bias else None) for w, b in P["conv"]]
    fcq = [(quantize(w, dtype), synth.round_f32(b).astype(np.float64)) for w, b in P["fc"]]
    xq, tq = quantize(x, dtype), synth.round_f32(t).astype(np.float64)
    net = CosmoFlowStack(to_dev(xq, dtype), to_dev(tq, "f32"),
                         [(to_dev(w, dtype), to_dev(b, "f32") if b is not None else None) for w, b in convq],
                         [(to_dev(w, dtype), to_dev(b, "f32")) for w, b in fcq], fuse_pool=fuse_pool, strides=strides, pools=pools)
    return net, xq, tq, convq, fcq


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-5), ("bf16", 2e-2)])
def test_cosmoflow_stack_miniature(dtype, tol):
    """3 stages on 32^3, batch 2: the full oracle runs in seconds."""
    import torch
    net, xq, tq, convq, fcq = build(dtype, 2, 32, (4, 16, 32, 64), (128, 32, 4), synth.BASE_SEED + 5)
    net.step()
    torch.cuda.synchronize()
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=lambda v: quantize(v, dtype))
    for i in range(len(convq)):
        assert rel_l2(from_dev(net.z[i].t), ref["z"][i].a) <= tol, f"z{i}"
    assert rel_l2(from_dev(net.y[-1]), ref["y"][-1]) <= tol
    assert abs(net.loss.item() - ref["loss"]) <= 4 * tol * abs(ref["loss"])
    # The loss gradient 2(pred - target)/count amplifies a one-ulp difference in pred by
    # |pred| / |pred - target|, and every gradient below is linear in it: the backward chain is
    # therefore started from the oracle's loss gradient on both sides (the MSE call itself is
    # compared on identical inputs in test_dense_and_mse).
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    # the masks are taken from each side's own z, so a few voxels near zero flip sign;
    # with slope 0.01 that perturbs the gradient norm far below the bar
    for i in range(len(fcq)):
        assert rel_l2(from_dev(net.dfc[i][0]), ref["dfc"][i][0]) <= 2 * tol, f"dfc{i}"
    for i in range(len(convq)):
        assert rel_l2(from_dev(net.dconv[i][0]), ref["dconv"][i][0]) <= 2 * tol, f"dw{i}"
        assert rel_l2(from_dev(net.dconv[i][1]), ref["dconv"][i][1]) <= 2 * tol, f"db{i}"
    assert rel_l2(from_dev(net.dx.t), ref["dx"].a) <= 2 * tol


def test_cosmoflow_stack_miniature_with_fused_first_stage():
    """The same miniature with the first stage's unpooled activation never stored (fused conv + pool forward, sign mask,
    pooling backward from the mask): same bars against the oracle; the first stage has no z to compare."""
    import torch
    dtype, tol = "bf16", 2e-2
    net, xq, tq, convq, fcq = build(dtype, 2, 32, (4, 16, 32, 64), (128, 32, 4), synth.BASE_SEED + 5, fuse_pool=True)
    assert net.fused == [True, False, False] and net.z[0] is None
    assert [o["name"] for o in net.ops][:3] == ["conv1_fwd_pool", "conv2_fwd", "pool2_fwd"]
    net.step()
    torch.cuda.synchronize()
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=lambda v: quantize(v, dtype))
    for i in range(1, len(convq)):
        assert rel_l2(from_dev(net.z[i].t), ref["z"][i].a) <= tol, f"z{i}"
    assert rel_l2(from_dev(net.y[-1]), ref["y"][-1]) <= tol
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    for i in range(len(convq)):
        assert rel_l2(from_dev(net.dconv[i][0]), ref["dconv"][i][0]) <= 2 * tol, f"dw{i}"
        assert rel_l2(from_dev(net.dconv[i][1]), ref["dconv"][i][1]) <= 2 * tol, f"db{i}"
    assert rel_l2(from_dev(net.dx.t), ref["dx"].a) <= 2 * tol
    # the same backward with the late backward-filter calls on a second stream: identical bits, several times over
    serial = [(dw.clone(), db.clone()) for dw, db in net.dconv]
    dx_serial = net.dx.t.clone()
    net.overlap = True
    for _ in range(3):
        for dw, db in net.dconv:
            dw.fill_(7.0)
            db.fill_(7.0)
        net.backward_after_loss()
        torch.cuda.synchronize()
        for (dw, db), (dw0, db0) in zip(net.dconv, serial):
            assert torch.equal(dw, dw0) and torch.equal(db, db0)
        assert torch.equal(net.dx.t, dx_serial)


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-5), ("bf16", 2e-2)])
def test_table1_shaped_miniature(dtype, tol):
    """The layer pattern of Table I on a 32^3 miniature, without convolution biases (Sec. IV): two stride-1 stages with
    pooling, a stride-2 convolution with pooling, a convolution on the remaining 2^3 volume without pooling, flatten,
    dense head."""
    import torch
    strides, pools = (1, 1, 2, 1), (True, True, True, False)
    net, xq, tq, convq, fcq = build(dtype, 2, 32, (4, 16, 32, 64, 64), (64, 16, 4), synth.BASE_SEED + 6, fuse_pool=True,
                                    strides=strides, pools=pools, flat_w=64 * 8, bias=False)
    assert [o["name"] for o in net.ops if "fwd" in o["name"]][-7:-2] == ["pool2_fwd", "conv3_fwd", "pool3_fwd", "conv4_fwd", "fc1_fwd"]
    net.step()
    torch.cuda.synchronize()
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=lambda v: quantize(v, dtype), strides=strides, pools=pools)
    for i in range(len(convq)):
        if net.z[i] is not None:
            assert rel_l2(from_dev(net.z[i].t), ref["z"][i].a) <= tol, f"z{i}"
    assert rel_l2(from_dev(net.y[-1]), ref["y"][-1]) <= tol
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    for i in range(len(convq)):
        assert rel_l2(from_dev(net.dconv[i][0]), ref["dconv"][i][0]) <= 2 * tol, f"dw{i}"
        assert net.dconv[i][1] is None
    assert rel_l2(from_dev(net.dx.t), ref["dx"].a) <= 2 * tol


@pytest.mark.parametrize("dg,d,d_offset,hw", [(32, 8, 0, 32), (32, 8, 8, 32), (32, 8, 24, 32), (64, 16, 16, 64)])
def test_unet_level_miniature(dg, d, d_offset, hw):
    """The U-Net-shaped level on linearly reduced shards (8x32x32 of a 32^3 volume: first, interior and
    last shard; 16x64x64 of a 64^3 volume = the 4x reduction of the real shard), 2-plane halo, full
    oracle, forward and backward, bf16."""
    import torch
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import UNetLevel
    from oracle_nets import unet_level_oracle
    dtype, tol = "bf16", 2e-2
    x, P, dout, faces = recipes.unet_level_inputs(synth.BASE_SEED + 9, d_global=dg, d=d, d_offset=d_offset, hw=hw)
    qz = lambda v: quantize(v, dtype)
    xq, doutq = qz(x), qz(dout)
    Pq = {k: (qz(w), synth.round_f32(b).astype(np.float64)) for k, (w, b) in P.items()}
    fq = {k: tuple(None if f is None else qz(f) for f in pair) for k, pair in faces.items()}
    Pd = {k: (to_dev(w, dtype), to_dev(b, "f32")) for k, (w, b) in Pq.items()}
    fd = {k: tuple(None if f is None else to_dev(f, dtype) for f in pair) for k, pair in fq.items()}
    net = UNetLevel(h3d.Slab(to_dev(xq, dtype), 2, 2, d_offset, dg), Pd, to_dev(doutq, dtype), fd)
    net.step()
    torch.cuda.synchronize()
    T, G, dP = unet_level_oracle(xq, 2, d_offset, dg, Pq, doutq, fq, q=qz)
    for k in ("a1", "a2", "p", "b1", "b2", "up", "cat", "out"):
        assert rel_l2(from_dev(net.T[k].t), T[k].a) <= tol, k
    assert np.array_equal(from_dev(net.T["cat"].t)[:, :, [0, -1]], T["cat"].a[:, :, [0, -1]])     # exchanged halo: bit-exact
    for k in ("g6", "dcat", "d_b2", "g4", "d_b1", "g3", "d_p", "d_a2", "g2", "d_a1", "g1", "dx"):
        assert rel_l2(from_dev(net.G[k].t), G[k].a) <= tol, k
    for k in dP:
        assert rel_l2(from_dev(net.dP[k][0]), dP[k][0]) <= tol, f"dw {k}"
        assert rel_l2(from_dev(net.dP[k][1]), dP[k][1]) <= tol, f"db {k}"


@pytest.mark.parametrize("d_offset", [0, 8, 24])
def test_cosmoflow_shard_chain_miniature(d_offset):
    """The spatially-partitioned front of the Table I network (three conv + pool stages with halo faces between them)
    on boundary and interior shards of a 4-way partitioned 32 x 32 x 32 sample, batch 2, bf16."""
    import torch
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import CosmoFlowShardChain
    dtype, tol = "bf16", 2e-2
    x, conv, dout, faces = recipes.shard_chain_inputs(synth.BASE_SEED + 7, 32, 8, d_offset, 32, (4, 16, 32, 64), n=2)
    qz = lambda v: None if v is None else quantize(v, dtype)
    xq, doutq = qz(x), qz(dout)
    convq = [(qz(w), None) for w, _ in conv]
    facesq = {k: (qz(lo), qz(hi)) for k, (lo, hi) in faces.items()}
    dv = lambda v: None if v is None else to_dev(v, dtype)
    net = CosmoFlowShardChain(h3d.Slab(dv(xq), 1, 1, d_offset, 32), [(dv(w), None) for w, _ in convq], dv(doutq),
                              {k: (dv(lo), dv(hi)) for k, (lo, hi) in facesq.items()})
    assert net.z[0] is None and net.ops[1]["name"] == "conv1_fwd_pool"
    net.step()
    torch.cuda.synchronize()
    ref = shard_chain_oracle(xq, d_offset, 32, convq, doutq, facesq, q=lambda v: quantize(v, dtype))
    for i in range(1, 4):
        assert rel_l2(from_dev(net.a[i].t), ref["a"][i].a) <= tol, f"a{i}"
    for i in range(3):
        assert rel_l2(from_dev(net.g[i].t), ref["g"][i].a) <= 2 * tol, f"g{i}"
        assert rel_l2(from_dev(net.dconv[i][0]), ref["dconv"][i][0]) <= 2 * tol, f"dw{i}"
        assert rel_l2(from_dev(net.da[i].t), ref["da"][i].a) <= 2 * tol, f"da{i}"
    # what this shard sends: the outermost interior planes of the pooled tensors and of the gradients
    for name, t in (("a1", ref["a"][1]), ("g1", ref["g"][0])):
        lo = from_dev(net.sent[name][0]).reshape(t.a[:, :, 1:2].shape)
        assert rel_l2(lo, t.a[:, :, 1:2]) <= 2 * tol
