"""The same network graphs evaluated with the CPU oracle (fp64), for the stack parity tests."""
from __future__ import annotations

import numpy as np

import oracle as orc


def cosmoflow_oracle(x, target, conv_params, fc_params, alpha=0.01, count=None, q=None, strides=None, pools=None):
    """Forward + backward of the CosmoFlow-shaped stack.  `q` rounds every STORED activation and
    activation gradient to the storage type (bf16 in / fp32 accumulate / bf16 out is the arithmetic
    contract of each layer, so a stack stores rounded tensors between layers); all sums stay fp64.  `count`: number of entries the MSE mean runs
    over (defaults to target.size; pass the full batch's count when evaluating a subset of samples)."""
    if q is None:
        q = lambda a: a
    qs = lambda s: orc.Slab(q(s.a), s.halo_lo, s.halo_hi, s.d_offset, s.d_global)
    xs = orc.Slab(x)
    strides = strides or [1] * len(conv_params)
    pools = pools or [True] * len(conv_params)
    cur, zs, ps, outs = xs, [], [], []
    for i, (w, b) in enumerate(conv_params):
        if strides[i] == 2:
            z = qs(orc.conv3d_s2_fwd(cur, w, b, orc.ACT_LEAKY, alpha))
        else:
            z = qs(orc.conv3d_fwd(cur, w, b, act=orc.ACT_LEAKY, alpha=alpha))
        p = qs(orc.pool3d_fwd(z, orc.POOL_AVG)) if pools[i] else None
        zs.append(z)
        ps.append(p)
        cur = p if p is not None else z
        outs.append(cur)
    n = x.shape[0]
    h = cur.a.reshape(n, -1)
    hs, ys = [h], []
    last = len(fc_params) - 1
    for i, (w, b) in enumerate(fc_params):
        h = q(orc.dense_fwd(h, w, b, orc.ACT_NONE if i == last else orc.ACT_LEAKY, alpha))
        ys.append(h)
        hs.append(h)
    loss, g = orc.mse_fwd_bwd(ys[-1], target)
    if count is not None:
        loss, g = loss * target.size / count, g * target.size / count
    dpred = q(g)

    def backward(g):
        """BD / BF of every layer from the loss gradient g [n, outputs]; linear in g (the masks come from the forward)."""
        dfc = [None] * len(fc_params)
        for i in range(last, -1, -1):
            g, dw, db = orc.dense_bwd(hs[i], fc_params[i][0], ys[i], g, orc.ACT_NONE if i == last else orc.ACT_LEAKY, alpha)
            dfc[i] = (dw, db)
            g = q(g)
        dp = orc.Slab(g.reshape(outs[-1].a.shape))
        dconv = [None] * len(conv_params)
        gs = [None] * len(conv_params)
        dps = [None] * len(conv_params)
        for i in range(len(conv_params) - 1, -1, -1):
            dps[i] = dp
            # pooling backward and activation backward form one stored tensor g (rounded once); without a pooling the
            # stored tensor is dz and the activation derivative is applied inside the two backward convolutions
            dz = orc.pool3d_bwd(dp, None, orc.POOL_AVG) if pools[i] else dp
            g = orc.act_bwd(dz, None, zs[i], orc.ACT_LEAKY, alpha)
            if pools[i]:
                g = qs(g)
            gs[i] = g
            xin = xs if i == 0 else outs[i - 1]
            if strides[i] == 2:
                dconv[i] = orc.conv3d_s2_bwd_filter(xin, g, None)
                dp = qs(orc.conv3d_s2_bwd_data(g, None, conv_params[i][0], xin))
            else:
                dconv[i] = orc.conv3d_bwd_filter(xin, g, None)
                dp = qs(orc.conv3d_bwd_data(g, None, conv_params[i][0]))
        return {"dfc": dfc, "dconv": dconv, "g": gs, "dx": dp, "dp": dps}

    out = {"z": zs, "p": ps, "out": outs, "y": ys, "loss": loss, "dpred": dpred, "backward": backward}
    out.update(backward(dpred))
    return out


def unet_level_oracle(x, halo, d_offset, d_global, P, dout, faces, q=None):
    """The U-Net-shaped level (same graph as paper_2007_12856_amd.nets.UNetLevel) with the oracle.
    x: [1,1,d+2*halo,H,W] float64; P: name -> (w, b); faces: name -> (lo, hi) arrays or None."""
    if q is None:
        q = lambda a: a
    R, NONE = orc.ACT_RELU, orc.ACT_NONE
    qs = lambda s: orc.Slab(q(s.a), s.halo_lo, s.halo_hi, s.d_offset, s.d_global)

    def with_halo(s, name, width):
        """re-home the interior of `s` in a slab with `width` halo planes filled by the exchange"""
        n, c, _, h, w = s.a.shape
        t = orc.Slab(np.zeros((n, c, s.d + 2 * width, h, w)), width, width, s.d_offset, s.d_global)
        t.interior[...] = s.interior
        lo, hi = faces[name]
        orc.halo_unpack(lo, t, orc.FACE_D_LO, width)
        orc.halo_unpack(hi, t, orc.FACE_D_HI, width)
        return t

    xs = orc.Slab(x, halo, halo, d_offset, d_global)
    T, G, dP = {}, {}, {}
    T["a1"] = qs(orc.conv3d_fwd(xs, *P["c1"], cout_halo=(1, 1), act=R))
    T["a2"] = qs(orc.conv3d_fwd(T["a1"], *P["c2"], act=R))
    T["p"] = with_halo(qs(orc.pool3d_fwd(T["a2"], orc.POOL_MAX)), "p", 2)
    T["b1"] = qs(orc.conv3d_fwd(T["p"], *P["c3"], cout_halo=(1, 1), act=R))
    T["b2"] = qs(orc.conv3d_fwd(T["b1"], *P["c4"], act=R))
    T["up"] = qs(orc.deconv2_fwd(T["b2"], *P["up"]))
    T["cat"] = with_halo(orc.concat_c(T["a2"], T["up"]), "cat", 1)
    T["out"] = qs(orc.conv3d_fwd(T["cat"], *P["c6"], act=R))
    dsl = orc.Slab(dout, 0, 0, d_offset, d_global)
    G["g6"] = with_halo(qs(orc.act_bwd(dsl, None, T["out"], R)), "g6", 1)
    dP["c6"] = orc.conv3d_bwd_filter(T["cat"], G["g6"], None)
    G["dcat"] = qs(orc.conv3d_bwd_data(G["g6"], None, P["c6"][0]))
    G["d_skip"], G["d_up"] = orc.split_c(G["dcat"], 64)
    dP["up"] = orc.deconv2_bwd_filter(T["b2"], G["d_up"])
    G["d_b2"] = qs(orc.deconv2_bwd_data(G["d_up"], P["up"][0]))
    G["g4"] = with_halo(qs(orc.act_bwd(G["d_b2"], None, T["b2"], R)), "g4", 1)
    dP["c4"] = orc.conv3d_bwd_filter(T["b1"], G["g4"], None)
    G["d_b1"] = qs(orc.conv3d_bwd_data(G["g4"], None, P["c4"][0]))
    G["g3"] = with_halo(qs(orc.act_bwd(G["d_b1"], None, T["b1"], R)), "g3", 1)
    dP["c3"] = orc.conv3d_bwd_filter(T["p"], G["g3"], None)
    G["d_p"] = qs(orc.conv3d_bwd_data(G["g3"], None, P["c3"][0]))
    G["d_a2"] = qs(orc.pool3d_bwd(G["d_p"], T["a2"], orc.POOL_MAX))
    G["g2"] = with_halo(qs(orc.act_bwd(G["d_a2"], G["d_skip"], T["a2"], R)), "g2", 1)
    dP["c2"] = orc.conv3d_bwd_filter(T["a1"], G["g2"], None)
    G["d_a1"] = qs(orc.conv3d_bwd_data(G["g2"], None, P["c2"][0]))
    G["g1"] = with_halo(qs(orc.act_bwd(G["d_a1"], None, T["a1"], R)), "g1", 1)
    dP["c1"] = orc.conv3d_bwd_filter(xs, G["g1"], None)
    G["dx"] = qs(orc.conv3d_bwd_data(G["g1"], None, P["c1"][0]))
    return T, G, dP


def shard_chain_oracle(x, d_offset, d_global, conv_params, dout, faces, alpha=0.01, q=None):
    """The chain of paper_2007_12856_amd.nets.CosmoFlowShardChain with the oracle.  x: [n,c,d+2,H,W] float64."""
    if q is None:
        q = lambda a: a
    qs = lambda s: orc.Slab(q(s.a), s.halo_lo, s.halo_hi, s.d_offset, s.d_global)

    def with_halo(s, name):
        n, c, _, h, w = s.a.shape
        t = orc.Slab(np.zeros((n, c, s.d + 2, h, w)), 1, 1, s.d_offset, s.d_global)
        t.interior[...] = s.interior
        lo, hi = faces[name]
        orc.halo_unpack(lo, t, orc.FACE_D_LO, 1)
        orc.halo_unpack(hi, t, orc.FACE_D_HI, 1)
        return t

    L = len(conv_params)
    a = [with_halo(orc.Slab(x, 1, 1, d_offset, d_global), "a0")]
    zs = []
    for i, (w, b) in enumerate(conv_params):
        z = qs(orc.conv3d_fwd(a[i], w, b, act=orc.ACT_LEAKY, alpha=alpha))
        p = qs(orc.pool3d_fwd(z, orc.POOL_AVG))
        zs.append(z)
        a.append(with_halo(p, f"a{i + 1}") if i < L - 1 else p)
    dp = orc.Slab(dout, 0, 0, a[L].d_offset, a[L].d_global)
    dconv, gs, da = [None] * L, [None] * L, [None] * L
    for i in range(L - 1, -1, -1):
        g = with_halo(qs(orc.act_bwd(orc.pool3d_bwd(dp, None, orc.POOL_AVG), None, zs[i], orc.ACT_LEAKY, alpha)), f"g{i + 1}")
        gs[i] = g
        dconv[i] = orc.conv3d_bwd_filter(a[i], g, None)
        dp = qs(orc.conv3d_bwd_data(g, None, conv_params[i][0]))
        da[i] = dp
    return {"a": a, "z": zs, "g": gs, "dconv": dconv, "da": da}
