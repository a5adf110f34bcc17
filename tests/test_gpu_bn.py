"""GPU parity of the local batch-normalisation passes against the oracle: a slab in the middle of a taller
volume (halo planes hold other data and must be ignored), ragged sizes, both storage types, two shards whose
statistics are added on the host in place of the allreduce."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,halo", [((2, 5, 3, 7, 9), 1), ((1, 16, 4, 32, 40), 0), ((3, 3, 2, 130, 128), 2)])
def test_bn_passes_two_shards(shape, halo, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, C, D, H, W = shape
    Dg = 2 * D
    full = synth.flat("normal", SEED, 60, (N, C, Dg + 2 * halo, H, W)) * 1.5 + 0.3
    gfull = synth.flat("normal", SEED, 61, (N, C, Dg, H, W))
    gamma = synth.round_f32(synth.flat("uniform", SEED, 62, (C,), 0.5, 1.5)).astype(np.float64)
    beta = synth.round_f32(synth.flat("uniform", SEED, 63, (C,), -0.5, 0.5)).astype(np.float64)
    eps, count = 1e-5, N * Dg * H * W
    shards = []
    for k in range(2):
        # stored planes of shard k: its D interior planes plus `halo` planes on each side (real neighbours or padding)
        a = full[:, :, k * D:k * D + D + 2 * halo]
        xo, xg = slab_pair(a, dtype, (halo, halo), k * D, Dg)
        go, gg = slab_pair(gfull[:, :, k * D:(k + 1) * D], dtype, (0, 0), k * D, Dg)
        shards.append((xo, xg, go, gg))
    f32 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).cuda()
    # ---- statistics: per shard on the GPU, summed on the host (the allreduce)
    so = sum(orc.bn_stats(s[0])[0] for s in shards)
    sqo = sum(orc.bn_stats(s[0])[1] for s in shards)
    sg, sqg = torch.zeros(C, device="cuda"), torch.zeros(C, device="cuda")
    for xo, xg, _, _ in shards:
        s1, s2 = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
        h3d.bn_stats(xg, s1, s2)
        s1b, s2b = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
        h3d.bn_stats(xg, s1b, s2b)
        assert torch.equal(s1, s1b) and torch.equal(s2, s2b)          # fixed summation order
        po = orc.bn_stats(xo)
        close(from_dev(s1), po[0], 1e-5)
        close(from_dev(s2), po[1], 1e-5)
        sg += s1
        sqg += s2
    mean_o, invstd_o = orc.bn_finalize(so, sqo, count, eps)
    mean_g, invstd_g = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    h3d.bn_finalize(sg, sqg, count, eps, mean_g, invstd_g)
    assert np.allclose(from_dev(mean_g), mean_o, rtol=1e-4, atol=1e-5) and np.allclose(from_dev(invstd_g), invstd_o, rtol=1e-4)
    # from here on both sides use the ORACLE's statistics (rounded to fp32), so that each pass is compared on its own
    mean32, invstd32 = synth.round_f32(mean_o).astype(np.float64), synth.round_f32(invstd_o).astype(np.float64)
    md, isd, gd, bd = f32(mean32), f32(invstd32), f32(gamma), f32(beta)
    # ---- forward
    for xo, xg, _, _ in shards:
        yo = orc.bn_fwd(xo, mean32, invstd32, gamma, beta)
        yg = h3d.bn_fwd(xg, md, isd, gd, bd, dev_like(yo, dtype))
        close(from_dev(yg.t), yo.a, TOL[dtype])
    # ---- backward sums, then the data gradient with the sums over both shards
    sdy_o = sum(orc.bn_bwd_stats(s[2], s[0], mean32, invstd32)[0] for s in shards)
    sdx_o = sum(orc.bn_bwd_stats(s[2], s[0], mean32, invstd32)[1] for s in shards)
    for xo, xg, go, gg in shards:
        a1, a2 = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
        h3d.bn_bwd_stats(gg, xg, md, isd, a1, a2)
        po = orc.bn_bwd_stats(go, xo, mean32, invstd32)
        scale = np.sqrt(N * D * H * W)        # sums of zero-mean terms: compare against their natural size
        assert np.max(np.abs(from_dev(a1) - po[0])) <= 1e-4 * scale and np.max(np.abs(from_dev(a2) - po[1])) <= 1e-4 * scale
    sdy32, sdx32 = synth.round_f32(sdy_o).astype(np.float64), synth.round_f32(sdx_o).astype(np.float64)
    for xo, xg, go, gg in shards:
        dxo = orc.bn_bwd(go, xo, mean32, invstd32, gamma, sdy32, sdx32, count)
        dxg = h3d.bn_bwd(gg, xg, md, isd, gd, f32(sdy32), f32(sdx32), count, dev_like(dxo, dtype))
        close(from_dev(dxg.t), dxo.a, TOL[dtype])


def test_bn_rejects_mismatched_shards_and_small_workspace():
    import torch
    import paper_2007_12856_amd as h3d
    _, xg = slab_pair(synth.flat("normal", SEED, 64, (1, 2, 4, 4, 8)), "bf16")
    _, yg = slab_pair(np.zeros((1, 3, 4, 4, 8)), "bf16")
    m = torch.zeros(2, device="cuda")
    with pytest.raises(h3d.H3DError):
        h3d.bn_fwd(xg, m, m, None, None, yg)
    with pytest.raises(h3d.H3DError):
        h3d._check(h3d.lib().h3d_bn_stats(h3d.handle(), __import__("ctypes").byref(xg.desc()), h3d._ptr(m), h3d._ptr(m), None, 0, None))
