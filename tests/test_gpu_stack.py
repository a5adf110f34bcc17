"""Whole-stack parity: the CosmoFlow-shaped network (conv+leaky+avg-pool stages, dense head, MSE),
forward and backward, HIP path vs the oracle on identical seeded bf16/fp32 inputs."""
import numpy as np
import pytest

import synth
from synth import recipes
from helpers import from_dev, quantize, close, rel_l2, to_dev
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


# Mask flips.  Each side takes the (leaky-)ReLU derivative from the sign of ITS OWN stored activation (the storage format
# is part of a layer's contract), so where an activation is within rounding of zero the two sides may pick different
# slopes: the gradient g at that voxel is then off by up to 0.99 |dz| on a fraction of voxels of the order of the
# relative rounding error, and every tensor downstream of it carries a small share of that.  The relative-L2 bar is
# unaffected (the flips perturb the norm far below it); the element-by-element check of the BACKWARD tensors of a stack
# therefore uses a wider factor and tolerates a small fraction of elements outside it (a wrong row or column of the
# miniatures is 3 % of a plane, of the full-size volumes 0.8 %).
BWD_ELEM = {"f32": dict(elem=1e-3, outliers=2e-3), "bf16": dict(elem=2.0 ** -4, outliers=2e-3)}
# Forward tensors of a stack differ by accumulated storage roundings of the layers before them (each side rounds its own
# sums): one bf16 ulp of an element's own rounding plus the propagated part.
FWD_ELEM = {"f32": dict(elem=1e-5), "bf16": dict(elem=2.0 ** -6)}


def loss_bound(pred_ref, target, tol):
    """|loss_gpu - loss_ref| / loss_ref for a prediction within relative L2 `tol` of the oracle's: the loss is
    mean (pred - t)^2, so d loss = 2 mean((pred - t) dpred) <= 2 |pred - t| |dpred| / count (Cauchy-Schwarz), i.e.
    2 tol |pred| / |pred - t| of the loss itself, to first order; the second-order term tol^2 |pred|^2 / |pred - t|^2 is added."""
    amp = np.linalg.norm(pred_ref) / np.linalg.norm(pred_ref - target)
    return 2 * tol * amp + (tol * amp) ** 2 + 1e-6


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-5), ("bf16", 2e-2)])
def test_cosmoflow_stack_miniature(dtype, tol):
    """3 stages on 32^3, batch 2: the full oracle runs in seconds.  Forward, loss, then the backward pass started from the
    ORACLE's loss gradient on both sides, so that every backward tensor is compared on its own bar (the unbroken chain
    is test_cosmoflow_stack_miniature_unbroken_chain)."""
    import torch
    net, xq, tq, convq, fcq = build(dtype, 2, 32, (4, 16, 32, 64), (128, 32, 4), synth.BASE_SEED + 5)
    net.step()
    torch.cuda.synchronize()
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=lambda v: quantize(v, dtype))
    for i in range(len(convq)):
        close(from_dev(net.z[i].t), ref["z"][i].a, tol, f"z{i}", **FWD_ELEM[dtype])
        close(from_dev(net.p[i].t), ref["p"][i].a, tol, f"p{i}", **FWD_ELEM[dtype])
    close(from_dev(net.y[-1]), ref["y"][-1], tol, "pred")
    assert abs(net.loss.item() - ref["loss"]) <= loss_bound(ref["y"][-1], tq, tol) * abs(ref["loss"])
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    for i in range(len(fcq)):
        close(from_dev(net.dfc[i][0]), ref["dfc"][i][0], tol, f"dfc{i}", **BWD_ELEM[dtype])
        close(from_dev(net.dfc[i][1]), ref["dfc"][i][1], tol, f"dfc{i} bias", **BWD_ELEM[dtype])
    for i in range(len(convq)):
        close(from_dev(net.g[i].t), ref["g"][i].a, tol, f"g{i}", **BWD_ELEM[dtype])
        close(from_dev(net.dconv[i][0]), ref["dconv"][i][0], tol, f"dw{i}", **BWD_ELEM[dtype])
        close(from_dev(net.dconv[i][1]), ref["dconv"][i][1], tol, f"db{i}", **BWD_ELEM[dtype])
    close(from_dev(net.dx.t), ref["dx"].a, tol, "dx", **BWD_ELEM[dtype])


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-5), ("bf16", 2e-2)])
def test_cosmoflow_stack_miniature_unbroken_chain(dtype, tol):
    """Forward -> MSE -> backward in one go, the backward pass fed by the GPU's OWN loss gradient (FP, then BD and BF of
    every layer, Sec. III-C, through the whole network).  The loss gradient 2 (pred - t) / count turns a relative
    difference e of pred into e |pred| / |pred - t| of itself, and every gradient is linear in it.  The bound is taken
    from that, in the test: with d = dpred_gpu - dpred_oracle (n x 4 numbers), the oracle's backward pass is run once per
    unit loss gradient (its Jacobian, columns J_j, from oracle inputs only), and a gradient tensor T must satisfy
    |T_gpu - T_oracle| <= tol |T_oracle| + |sum_j d_j J_j(T)| (1 + tol): the GPU's own error on the bar, plus what the
    different starting point explains."""
    import torch
    n = 2
    net, xq, tq, convq, fcq = build(dtype, n, 32, (4, 16, 32, 64), (128, 32, 4), synth.BASE_SEED + 5, fuse_pool=(dtype == "bf16"))
    net.step()                                             # one unbroken pass: no tensor is touched between the calls
    torch.cuda.synchronize()
    ref = cosmoflow_oracle(xq, tq, convq, fcq, q=lambda v: quantize(v, dtype))
    pred_ref, dpred_ref = ref["y"][-1], ref["dpred"]
    close(from_dev(net.y[-1]), pred_ref, tol, "pred")
    amp = np.linalg.norm(pred_ref) / np.linalg.norm(pred_ref - tq)
    dpred_gpu = from_dev(net.dy[-1])
    # storage rounding of dpred (one per side) on top of the amplified difference of pred
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    assert rel_l2(dpred_gpu, dpred_ref) <= tol * amp + 2 * ulp, "loss gradient"
    delta = dpred_gpu - dpred_ref
    # Jacobian of the oracle's backward pass with respect to the loss gradient
    basis = []
    for j in range(delta.size):
        e = np.zeros(delta.size)
        e[j] = 1.0
        basis.append(ref["backward"](e.reshape(delta.shape)))

    def explained(pick):
        return sum(float(delta.flat[j]) * np.asarray(pick(basis[j])) for j in range(delta.size))

    def bounded(got, pick, what):
        want = np.asarray(pick(ref))
        lim = tol * np.linalg.norm(want) + (1 + tol) * np.linalg.norm(explained(pick))
        err = np.linalg.norm(np.asarray(got, dtype=np.float64) - want)
        assert err <= lim, f"{what}: |gpu - oracle| {err:.3e} > {lim:.3e} (|oracle| {np.linalg.norm(want):.3e})"
        # and against the oracle's result moved to the GPU's starting point, element by element
        close(got, want + explained(pick), tol, what, **BWD_ELEM[dtype])

    for i in range(len(fcq)):
        bounded(from_dev(net.dfc[i][0]), lambda r, i=i: r["dfc"][i][0], f"dfc{i}")
        bounded(from_dev(net.dfc[i][1]), lambda r, i=i: r["dfc"][i][1], f"dfc{i} bias")
    for i in range(len(convq)):
        bounded(from_dev(net.g[i].t), lambda r, i=i: r["g"][i].a, f"g{i}")
        bounded(from_dev(net.dconv[i][0]), lambda r, i=i: r["dconv"][i][0], f"dw{i}")
        bounded(from_dev(net.dconv[i][1]), lambda r, i=i: r["dconv"][i][1], f"db{i}")
    bounded(from_dev(net.dx.t), lambda r: r["dx"].a, "dx")


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
        close(from_dev(net.z[i].t), ref["z"][i].a, tol, f"z{i}", **FWD_ELEM[dtype])
    close(from_dev(net.y[-1]), ref["y"][-1], tol, "pred")
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    for i in range(len(convq)):
        close(from_dev(net.dconv[i][0]), ref["dconv"][i][0], tol, f"dw{i}", **BWD_ELEM[dtype])
        close(from_dev(net.dconv[i][1]), ref["dconv"][i][1], tol, f"db{i}", **BWD_ELEM[dtype])
    close(from_dev(net.dx.t), ref["dx"].a, tol, "dx", **BWD_ELEM[dtype])
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
            close(from_dev(net.z[i].t), ref["z"][i].a, tol, f"z{i}", **FWD_ELEM[dtype])
    close(from_dev(net.y[-1]), ref["y"][-1], tol, "pred")
    net.dy[-1].copy_(to_dev(ref["dpred"], dtype))
    net.backward_after_loss()
    torch.cuda.synchronize()
    for i in range(len(convq)):
        close(from_dev(net.dconv[i][0]), ref["dconv"][i][0], tol, f"dw{i}", **BWD_ELEM[dtype])
        assert net.dconv[i][1] is None
    close(from_dev(net.dx.t), ref["dx"].a, tol, "dx", **BWD_ELEM[dtype])


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
        close(from_dev(net.T[k].t), T[k].a, tol, k, **FWD_ELEM[dtype])
    assert np.array_equal(from_dev(net.T["cat"].t)[:, :, [0, -1]], T["cat"].a[:, :, [0, -1]])     # exchanged halo: bit-exact
    assert "concat" not in [o["name"] for o in net.ops] and "split" not in [o["name"] for o in net.ops]     # views, no copies
    assert net.T["a2"].t.data_ptr() == net.T["cat"].interior.data_ptr()
    for k in ("g6", "dcat", "d_b2", "g4", "d_b1", "g3", "d_p", "g2", "d_a1", "g1", "dx"):
        close(from_dev(net.G[k].t), G[k].a, tol, k, **BWD_ELEM[dtype])
    for k in dP:
        close(from_dev(net.dP[k][0]), dP[k][0], tol, f"dw {k}", **BWD_ELEM[dtype])
        close(from_dev(net.dP[k][1]), dP[k][1], tol, f"db {k}", **BWD_ELEM[dtype])


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
        close(from_dev(net.a[i].t), ref["a"][i].a, tol, f"a{i}", **FWD_ELEM[dtype])
    for i in range(3):
        close(from_dev(net.g[i].t), ref["g"][i].a, tol, f"g{i}", **BWD_ELEM[dtype])
        close(from_dev(net.dconv[i][0]), ref["dconv"][i][0], tol, f"dw{i}", **BWD_ELEM[dtype])
        close(from_dev(net.da[i].t), ref["da"][i].a, tol, f"da{i}", **BWD_ELEM[dtype])
    # what this shard sends: the outermost interior planes of the pooled tensors and of the gradients
    for name, t in (("a1", ref["a"][1]), ("g1", ref["g"][0])):
        lo = from_dev(net.sent[name][0]).reshape(t.a[:, :, 1:2].shape)
        close(lo, t.a[:, :, 1:2], tol, name, **BWD_ELEM[dtype])
