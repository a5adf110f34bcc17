"""The same network graphs evaluated with the CPU oracle (fp64), for the stack parity tests."""
from __future__ import annotations

import numpy as np

import oracle as orc


def cosmoflow_oracle(x, target, conv_params, fc_params, alpha=0.01, count=None, q=None):
    """Forward + backward of the CosmoFlow-shaped stack.  `q` rounds every STORED activation and
    activation gradient to the storage type (bf16 in / fp32 accumulate / bf16 out is the arithmetic
    contract of each layer, so a stack stores rounded tensors between layers); all sums stay fp64.  `count`: number of entries the MSE mean runs
    over (defaults to target.size; pass the full batch's count when evaluating a subset of samples)."""
    if q is None:
        q = lambda a: a
    qs = lambda s: orc.Slab(q(s.a), s.halo_lo, s.halo_hi, s.d_offset, s.d_global)
    xs = orc.Slab(x)
    cur, zs, ps = xs, [], []
    for w, b in conv_params:
        z = qs(orc.conv3d_fwd(cur, w, b, act=orc.ACT_LEAKY, alpha=alpha))
        p = qs(orc.pool3d_fwd(z, orc.POOL_AVG))
        zs.append(z)
        ps.append(p)
        cur = p
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
    g = q(g)
    dfc = [None] * len(fc_params)
    for i in range(last, -1, -1):
        g, dw, db = orc.dense_bwd(hs[i], fc_params[i][0], ys[i], g, orc.ACT_NONE if i == last else orc.ACT_LEAKY, alpha)
        dfc[i] = (dw, db)
        g = q(g)
    dp = orc.Slab(g.reshape(ps[-1].a.shape))
    dconv = [None] * len(conv_params)
    dzs = [None] * len(conv_params)
    for i in range(len(conv_params) - 1, -1, -1):
        dz = qs(orc.pool3d_bwd(dp, None, orc.POOL_AVG))
        dzs[i] = dz
        xin = xs if i == 0 else ps[i - 1]
        dconv[i] = orc.conv3d_bwd_filter(xin, dz, zs[i], act=orc.ACT_LEAKY, alpha=alpha)
        dp = qs(orc.conv3d_bwd_data(dz, zs[i], conv_params[i][0], act=orc.ACT_LEAKY, alpha=alpha))
    return {"z": zs, "p": ps, "y": ys, "loss": loss, "dfc": dfc, "dconv": dconv, "dz": dzs, "dx": dp}
