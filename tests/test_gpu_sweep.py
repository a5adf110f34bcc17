"""Seeded sweep of small random shapes through the three convolution passes (with and without the fused activation
mask, with and without halos, packed and as plane-run views) and the transposed convolution, against the oracle.
The shapes are drawn so that every kernel family is reached: first-layer kernels (Cin <= 4), the few-channel
kernel (<= 8 output channels), 16/32-channel workgroups, narrow (W <= 16) and wide volumes, ragged H / W / channels."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    chans = [1, 2, 3, 4, 5, 8, 12, 16, 17, 24, 32, 33, 40, 48, 64, 72]
    widths = [4, 8, 12, 16, 24, 32, 33, 40, 48, 64, 72]
    out = []
    for i in range(n):
        cin, cout = int(rng.choice(chans)), int(rng.choice(chans))
        W = int(rng.choice(widths))
        H = int(rng.integers(2, 13)) if W > 16 else int(rng.integers(2, 20))
        D = int(rng.integers(1, 6))
        N = int(rng.integers(1, 3))
        halo = int(rng.integers(0, 2))
        # keep the oracle's direct loops under a second per case
        if N * D * H * W * cin * cout > 3_000_000:
            N, D = 1, min(D, 2)
        out.append((i, N, cin, cout, D, H, W, halo, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("case", _cases(36, 2007), ids=lambda c: "c%d_%dx%d-%d_%dx%dx%d_h%d_m%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8]))
def test_conv_sweep_bf16(case):
    import torch
    import paper_2007_12856_amd as h3d
    i, N, cin, cout, D, H, W, halo, masked = case
    dtype = "bf16"
    b = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, 1000 + i, (cout, cin, 3, 3, 3), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, 2000 + i, (cout,), -0.1, 0.1)).astype(np.float64)
    Dg, off = (D + 2, 1) if halo else (D, 0)
    xo, xg = slab_pair(synth.flat("normal", SEED, 3000 + i, (N, cin, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    act = orc.ACT_LEAKY if masked else orc.ACT_NONE
    zo = orc.conv3d_fwd(xo, w, bias, act=act, alpha=0.01)
    zg = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, dtype), act, 0.01)
    close(from_dev(zg.t), zo.a, TOL[dtype])
    # the backward passes take ANY saved output as the activation mask: a seeded one with the halo dz is read at
    zm_o, zm_g = slab_pair(synth.flat("normal", SEED, 6000 + i, (N, cout, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    zq_o, zq_g = slab_pair(zm_o.interior, dtype, (0, 0), off, Dg)
    # gradient of the layer's output with a halo of its own (neighbouring shards' planes), as backward-data needs it
    go, gg = slab_pair(synth.flat("normal", SEED, 4000 + i, (N, cout, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    if masked:
        dxo = orc.conv3d_bwd_data(go, zm_o, w, act=act, alpha=0.01)
        dxg = h3d.conv3d_bwd_data(gg, zm_g, wd, dev_like(dxo, dtype), act, 0.01)
    else:
        dxo = orc.conv3d_bwd_data(go, None, w, act=orc.ACT_NONE)
        dxg = h3d.conv3d_bwd_data(gg, None, wd, dev_like(dxo, dtype), h3d.ACT_NONE, 0.0)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    g0o, g0g = slab_pair(go.interior, dtype, (0, 0), off, Dg)
    dwo, dbo = orc.conv3d_bwd_filter(xo, g0o, zq_o if masked else None, act=act, alpha=0.01)
    dw = torch.full((cout, cin, 3, 3, 3), 7.0, device="cuda")
    db = torch.full((cout,), 7.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, g0g, zq_g if masked else None, dw, db, act, 0.01)
    close(from_dev(dw), dwo, 2e-4)
    close(from_dev(db), dbo, 2e-4)
    # the same forward on a plane-run view of the middle planes (when there are at least three)
    if D >= 3:
        part = dev_like(zo, dtype)
        part.t.zero_()
        h3d.conv3d_fwd(xg.planes(1, D - 1, 1, 1), wd, bd, part.planes(1, D - 1), act, 0.01)
        close(from_dev(part.t[:, :, 1:D - 1]), zo.a[:, :, 1:D - 1], TOL[dtype])
        assert float(part.t[:, :, 0].abs().max()) == 0.0 and float(part.t[:, :, D - 1].abs().max()) == 0.0


@pytest.mark.parametrize("case", [(0, 1, 8, 12, 2, 3, 8), (1, 2, 33, 7, 1, 5, 16), (2, 1, 64, 64, 2, 4, 24), (3, 1, 128, 32, 1, 2, 40),
                                  (4, 1, 96, 48, 2, 2, 8), (5, 2, 16, 16, 3, 6, 32)])
def test_deconv_sweep_bf16(case):
    import torch
    import paper_2007_12856_amd as h3d
    i, N, cin, cout, d, H, W = case
    dtype = "bf16"
    b = np.sqrt(3.0 / (8 * cin))
    w = quantize(synth.flat("uniform", SEED, 5000 + i, (cin, cout, 2, 2, 2), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, 5100 + i, (cout,), -0.1, 0.1)).astype(np.float64)
    xo, xg = slab_pair(synth.flat("normal", SEED, 5200 + i, (N, cin, d, H, W)), dtype, (0, 0), 1, d + 3)
    yo = orc.deconv2_fwd(xo, w, bias)
    yg = h3d.deconv2_fwd(xg, to_dev(w, dtype), to_dev(bias, "f32"), dev_like(yo, dtype))
    close(from_dev(yg.t), yo.a, TOL[dtype])
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 5300 + i, yo.a.shape), dtype, (0, 0), yo.d_offset, yo.d_global)
    dxo = orc.deconv2_bwd_data(dyo, w)
    dxg = h3d.deconv2_bwd_data(dyg, to_dev(w, dtype), dev_like(dxo, dtype))
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.deconv2_bwd_filter(xo, dyo)
    dw, db = torch.empty((cin, cout, 2, 2, 2), device="cuda"), torch.empty((cout,), device="cuda")
    h3d.deconv2_bwd_filter(xg, dyg, dw, db)
    close(from_dev(dw), dwo, 2e-4)
    close(from_dev(db), dbo, 2e-4)
