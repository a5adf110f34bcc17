"""GPU parity of the three convolution passes against the CPU oracle (relative L2 and an element-by-element bound), on
seeded inputs at sizes the oracle finishes in seconds: several tiles, ragged tails, odd channel
counts, boundary and interior shards, halo recompute.  All calls go through the C ABI."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, cut, dev_like, elem_masked_bf, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED

# (N, Cin, Cout, Dg, H, W)
SHAPES = [
    (1, 4, 16, 32, 32, 32),      # the single-layer fp32 configuration's shape
    (2, 3, 5, 6, 7, 9),          # nothing divides anything
    (1, 1, 32, 8, 20, 70),       # single input channel (U-Net first layer), W spans two 64-wide tiles raggedly
    (1, 17, 4, 5, 9, 33),
    (2, 16, 32, 8, 12, 40),
    (1, 32, 64, 6, 10, 36),
    (1, 64, 16, 4, 6, 66),
    (1, 8, 8, 1, 1, 1),          # degenerate volume
]


def _weights(cin, cout, dtype, stream):
    b = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, stream, (cout, cin, 3, 3, 3), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, stream + 1, (cout,), -0.1, 0.1)).astype(np.float64)
    return w, bias


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_conv3d_three_passes_unsharded(shape, dtype):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = shape
    alpha = 0.01
    w, bias = _weights(Ci, Co, dtype, 10)
    xo, xg = slab_pair(synth.flat("uniform", SEED, 1, (N, Ci, D, H, W)), dtype)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    # forward
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=alpha)
    zg = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(zg.t), zo.a, TOL[dtype])
    # backward passes take the ORACLE's z (rounded to storage) as the saved output on both sides
    zq_o, zq_g = slab_pair(zo.a, dtype)
    dzo, dzg = slab_pair(synth.flat("uniform", SEED, 2, (N, Co, D, H, W)), dtype)
    dxo = orc.conv3d_bwd_data(dzo, zq_o, w, act=orc.ACT_LEAKY, alpha=alpha)
    dxg = h3d.conv3d_bwd_data(dzg, zq_g, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, zq_o, act=orc.ACT_LEAKY, alpha=alpha)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, zq_g, dw, db, h3d.ACT_LEAKY, alpha)
    # dW stays fp32: with exact bf16 products and fp32 accumulation the error is far below the bf16 bar
    tol_w = 1e-5 if dtype == "f32" else 2e-4
    close(from_dev(dw), dwo, tol_w, elem=elem_masked_bf(dtype))
    close(from_dev(db), dbo, tol_w, elem=elem_masked_bf(dtype))
    # deterministic split-spatial reduction: a second call returns identical bits
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_bwd_filter(xg, dzg, zq_g, dw2, db2, h3d.ACT_LEAKY, alpha)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_RELU])
def test_conv3d_no_bias_and_other_activations(dtype, act):
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W = 1, 8, 16, 4, 6, 20
    w, _ = _weights(Ci, Co, dtype, 20)
    xo, xg = slab_pair(synth.flat("normal", SEED, 3, (N, Ci, D, H, W)), dtype)
    zo = orc.conv3d_fwd(xo, w, None, act=act)
    zg = h3d.conv3d_fwd(xg, to_dev(w, dtype), None, dev_like(zo, dtype), act, 0.0)
    close(from_dev(zg.t), zo.a, TOL[dtype])
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 4, (N, Co, D, H, W)), dtype)
    zq_o, zq_g = slab_pair(zo.a, dtype)
    dxo = orc.conv3d_bwd_data(dzo, zq_o, w, act=act)
    dxg = h3d.conv3d_bwd_data(dzg, zq_g, to_dev(w, dtype), dev_like(dxo, dtype), act, 0.0)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])


# (N, Cin, Cout, D, H, W, halo): unmasked filter gradients (the activation's mask already applied upstream), shapes
# chosen to reach every workgroup layout of the matrix-core kernels: first-layer (Cin <= 4) with one and two
# row blocks, 16- and 32-channel workgroups, one and two row groups, 4- and 6-row tiles, ragged H / W / channels
BF_SHAPES = [
    (1, 4, 16, 3, 36, 40, 1),
    (2, 3, 24, 2, 20, 64, 0),
    (1, 1, 40, 3, 33, 32, 1),
    (1, 16, 32, 3, 12, 40, 1),
    (1, 12, 16, 2, 9, 32, 0),
    (1, 32, 64, 3, 50, 32, 1),
    (1, 48, 80, 2, 10, 72, 1),
    (1, 20, 16, 2, 8, 96, 0),
    (1, 24, 24, 5, 7, 33, 1),
    (1, 4, 16, 2, 20, 72, 1),
    (1, 2, 10, 3, 17, 128, 0),
    # more than 32 channels on both sides: the kernel on the 32x32x16 tile (64-, 32- and 16-voxel row segments, ragged
    # bands and channel blocks, a ragged last K-step, chunks of several strips that cross planes and samples)
    (2, 40, 48, 3, 20, 16, 1),
    (1, 72, 40, 2, 9, 32, 0),
    (1, 64, 64, 4, 34, 64, 1),
    (2, 40, 40, 5, 18, 24, 1),
    (1, 36, 130, 2, 6, 136, 0),
    (4, 130, 130, 5, 10, 16, 1),
]


@pytest.mark.parametrize("kernel", ["by shape", "32x32x16 tile"])
@pytest.mark.parametrize("shape", BF_SHAPES)
def test_conv3d_bwd_filter_unmasked_bf16(shape, kernel, monkeypatch):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W, halo = shape
    if kernel == "32x32x16 tile":
        # the library gives volumes this small to the kernels with smaller workgroup tiles; H3D_BF_ROW32=1 lifts that
        # limit, so that the many-channel kernel is compared with the oracle at sizes the oracle finishes in seconds
        if not (Ci > 32 and Co > 32):
            pytest.skip("the kernel takes more than 32 channels on both sides")
        monkeypatch.setenv("H3D_BF_ROW32", "1")
    else:
        monkeypatch.delenv("H3D_BF_ROW32", raising=False)
    dtype = "bf16"
    # with halo: the middle slab of a volume two planes taller (the halo planes hold real neighbours);
    # without: the whole volume, zero beyond both ends
    Dg, off = (D + 2, 1) if halo else (D, 0)
    xo, xg = slab_pair(synth.flat("normal", SEED, 30, (N, Ci, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 31, (N, Co, D, H, W)), dtype, (0, 0), off, Dg)
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, None, act=orc.ACT_NONE)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, None, dw, db, h3d.ACT_NONE, 0.0)
    close(from_dev(dw), dwo, 2e-4)
    close(from_dev(db), dbo, 2e-4)
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_bwd_filter(xg, dzg, None, dw2, db2, h3d.ACT_NONE, 0.0)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)
    if kernel == "32x32x16 tile":
        assert h3d.h3d_last_kernel().startswith("bwd_filter_row32_kernel"), h3d.h3d_last_kernel()


def _row32_random_shapes(k=8):
    rng = np.random.default_rng(SEED + 77)
    out = []
    for _ in range(k):
        out.append((int(rng.integers(1, 4)), int(rng.integers(33, 81)), int(rng.integers(33, 81)), int(rng.integers(1, 6)),
                    int(rng.integers(1, 21)), int(rng.choice([16, 24, 32, 40, 48, 64, 72, 96])), int(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("shape", _row32_random_shapes())
def test_conv3d_bwd_filter_many_channels_random_shapes(shape, monkeypatch):
    """Seeded random shapes for the kernel on the 32x32x16 tile (test hook H3D_BF_ROW32, see above): ragged channel
    blocks, bands, K-steps and chunks in combinations nobody picked by hand."""
    import torch
    import paper_2007_12856_amd as h3d
    monkeypatch.setenv("H3D_BF_ROW32", "1")
    N, Ci, Co, D, H, W, halo = shape
    dtype = "bf16"
    Dg, off = (D + 2, 1) if halo else (D, 0)
    xo, xg = slab_pair(synth.flat("normal", SEED, 32, (N, Ci, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 33, (N, Co, D, H, W)), dtype, (0, 0), off, Dg)
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, None, act=orc.ACT_NONE)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, None, dw, db, h3d.ACT_NONE, 0.0)
    assert h3d.h3d_last_kernel().startswith("bwd_filter_row32_kernel"), h3d.h3d_last_kernel()
    close(from_dev(dw), dwo, 2e-4, f"dw {shape}")
    close(from_dev(db), dbo, 2e-4, f"db {shape}")


# (N, Cin, Cout, D, H, W, halo): layers with a handful of channels on one side and at most 16 on the other, wide
# enough for the tap-row-folding kernel: backward-data onto <= 8 channels (no fused mask), forward onto <= 8
THIN_SHAPES = [
    (1, 4, 16, 5, 9, 40, 1),
    (2, 3, 12, 3, 6, 66, 0),
    (1, 8, 16, 6, 10, 32, 1),
    (1, 1, 7, 2, 5, 130, 0),
    # at most 4 channels, W a multiple of 8, H >= 8: the row-streaming variant (several depth tiles with a ragged
    # last one, several row segments, one to three column tiles)
    (2, 4, 16, 7, 33, 136, 1),
    (1, 2, 9, 9, 8, 64, 0),
    (1, 3, 16, 4, 20, 72, 1),
    (1, 4, 12, 2, 70, 32, 1),
    # backward-data onto at most 4 channels from 17 to 32: two passes of the row-streaming kernel over channel halves
    (1, 1, 32, 5, 12, 72, 1),
    (2, 4, 24, 3, 9, 40, 0),
    (1, 2, 17, 4, 16, 136, 1),
]


@pytest.mark.parametrize("shape", THIN_SHAPES)
def test_conv3d_few_channels_bf16(shape):
    import paper_2007_12856_amd as h3d
    N, Cs, Cl, D, H, W, halo = shape      # Cs: the small channel count, Cl: the larger one
    dtype = "bf16"
    Dg, off = (D + 2, 1) if halo else (D, 0)
    # backward-data of a Cs -> Cl layer: dz has Cl channels and a halo, dx has Cs channels
    w, bias = _weights(Cs, Cl, dtype, 40)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 41, (N, Cl, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    dxo = orc.conv3d_bwd_data(dzo, None, w, act=orc.ACT_NONE)
    dxg = h3d.conv3d_bwd_data(dzg, None, to_dev(w, dtype), dev_like(dxo, dtype), h3d.ACT_NONE, 0.0)
    close(from_dev(dxg.t), dxo.a, TOL[dtype])
    # forward of a Cl -> Cs layer with bias and leaky ReLU
    w2, bias2 = _weights(Cl, Cs, dtype, 42)
    xo, xg = slab_pair(synth.flat("normal", SEED, 43, (N, Cl, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    zo = orc.conv3d_fwd(xo, w2, bias2, act=orc.ACT_LEAKY, alpha=0.01)
    zg = h3d.conv3d_fwd(xg, to_dev(w2, dtype), to_dev(bias2, "f32"), dev_like(zo, dtype), h3d.ACT_LEAKY, 0.01)
    close(from_dev(zg.t), zo.a, TOL[dtype])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cin,cout", [(4, 16), (3, 5), (16, 32)])
def test_conv3d_sharded_matches_oracle_and_unsharded_gpu(dtype, cin, cout):
    """Boundary and interior shards; halo planes outside the volume hold a canary that must not be read;
    the concatenated shard outputs equal the unsharded GPU output bit for bit (the accumulation
    order of a voxel does not depend on the slab it is computed in)."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Dg, H, W, nshard = 2, 12, 10, 34, 3
    d = Dg // nshard
    full = (N, cin, Dg, H, W)
    w, bias = _weights(cin, cout, dtype, 30)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    xfo, xfg = slab_pair(synth.slab("cosmo", SEED, 5, full, 0, Dg), dtype)
    zfo = orc.conv3d_fwd(xfo, w, bias, act=orc.ACT_LEAKY, alpha=0.01)
    zfg = h3d.conv3d_fwd(xfg, wd, bd, dev_like(zfo, dtype), h3d.ACT_LEAKY, 0.01)
    dzf = synth.slab("normal", SEED, 6, (N, cout, Dg, H, W), 0, Dg)
    dzfo, dzfg = slab_pair(dzf, dtype)
    zqo, zqg = slab_pair(zfo.a, dtype)
    dxfg = h3d.conv3d_bwd_data(dzfg, zqg, wd, dev_like(xfo, dtype), h3d.ACT_LEAKY, 0.01)
    dwf = torch.empty((cout, cin, 3, 3, 3), device="cuda")
    dbf = torch.empty((cout,), device="cuda")
    h3d.conv3d_bwd_filter(xfg, dzfg, zqg, dwf, dbf, h3d.ACT_LEAKY, 0.01)
    dw_sum = torch.zeros_like(dwf, dtype=torch.float64)
    db_sum = torch.zeros_like(dbf, dtype=torch.float64)
    dwo_sum = 0.0
    for s in range(nshard):
        off = s * d
        xs = cut("cosmo", SEED, 5, full, off, d, (1, 1))
        for pl, g in enumerate(range(off - 1, off + d + 1)):
            if g < 0 or g >= Dg:
                xs[:, :, pl] = 999.0          # canary outside the volume
        xo, xg = slab_pair(xs, dtype, (1, 1), off, Dg)
        zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=0.01)
        zg = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, dtype), h3d.ACT_LEAKY, 0.01)
        close(from_dev(zg.t), zo.a, TOL[dtype])
        assert torch.equal(zg.t, zfg.t[:, :, off:off + d])
        # backward-data: dz and z carry the exchanged halo
        zs = np.full((N, cout, d + 2, H, W), 999.0)
        dzs = np.full((N, cout, d + 2, H, W), 999.0)
        for pl, g in enumerate(range(off - 1, off + d + 1)):
            if 0 <= g < Dg:
                zs[:, :, pl], dzs[:, :, pl] = zfo.a[:, :, g], dzf[:, :, g]
        zso, zsg = slab_pair(zs, dtype, (1, 1), off, Dg)
        dzo, dzg = slab_pair(dzs, dtype, (1, 1), off, Dg)
        dxo = orc.conv3d_bwd_data(dzo, zso, w, act=orc.ACT_LEAKY, alpha=0.01)
        dxg = h3d.conv3d_bwd_data(dzg, zsg, wd, dev_like(dxo, dtype), h3d.ACT_LEAKY, 0.01)
        close(from_dev(dxg.t), dxo.a, TOL[dtype])
        assert torch.equal(dxg.t, dxfg.t[:, :, off:off + d])
        # backward-filter partial of this shard
        dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, zso, act=orc.ACT_LEAKY, alpha=0.01)
        dw, db = torch.empty_like(dwf), torch.empty_like(dbf)
        h3d.conv3d_bwd_filter(xg, dzg, zsg, dw, db, h3d.ACT_LEAKY, 0.01)
        close(from_dev(dw), dwo, TOL[dtype])
        close(from_dev(db), dbo, TOL[dtype])
        dw_sum += dw.double()
        db_sum += db.double()
        dwo_sum = dwo_sum + dwo
    close(dw_sum.cpu().numpy(), from_dev(dwf), 1e-5)
    close(db_sum.cpu().numpy(), from_dev(dbf), 1e-5)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cin,cout,W,exact", [(4, 16, 40, True), (16, 32, 32, True), (24, 8, 36, True), (64, 128, 40, True),
                                              (64, 128, 8, False)])
def test_main_halo_split_is_bit_exact(dtype, cin, cout, W, exact):
    """Sec. III-C: the planes that need no halo (main) and the two strips that do are computed by separate
    calls on plane-run views of the same buffers; together they must reproduce the whole-slab call bit for bit."""
    import torch
    import paper_2007_12856_amd as h3d
    N, D, H = 2, 9, 18
    w, bias = _weights(cin, cout, dtype, 50)
    wd, bd = to_dev(w, dtype), to_dev(bias, "f32")
    xo, xg = slab_pair(synth.flat("normal", SEED, 51, (N, cin, D + 2, H, W)), dtype, (1, 1), 3, D + 6)
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=0.01)
    whole = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, dtype), h3d.ACT_LEAKY, 0.01)
    close(from_dev(whole.t), zo.a, TOL[dtype])
    parts = dev_like(zo, dtype)
    for p0, p1 in [(1, D - 1), (0, 1), (D - 1, D)]:          # main first, then the two strips
        h3d.conv3d_fwd(xg.planes(p0, p1, 1, 1), wd, bd, parts.planes(p0, p1), h3d.ACT_LEAKY, 0.01)
    if exact or dtype == "f32":
        assert torch.equal(parts.t, whole.t)
    else:
        close(from_dev(parts.t), zo.a, TOL[dtype])
    # backward-data on the same split
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 52, (N, cout, D + 2, H, W)), dtype, (1, 1), 3, D + 6)
    dxo = orc.conv3d_bwd_data(dzo, None, w, act=orc.ACT_NONE)
    dx_whole = h3d.conv3d_bwd_data(dzg, None, wd, dev_like(dxo, dtype), h3d.ACT_NONE, 0.0)
    close(from_dev(dx_whole.t), dxo.a, TOL[dtype])
    dx_parts = dev_like(dxo, dtype)
    for p0, p1 in [(2, D - 2), (0, 2), (D - 2, D)]:
        h3d.conv3d_bwd_data(dzg.planes(p0, p1, 1, 1), None, wd, dx_parts.planes(p0, p1), h3d.ACT_NONE, 0.0)
    if exact or dtype == "f32":
        assert torch.equal(dx_parts.t, dx_whole.t)
    else:
        close(from_dev(dx_parts.t), dxo.a, TOL[dtype])
    # backward-filter: the strips' partial gradients add up to the whole slab's (different summation order)
    go, gg = slab_pair(synth.flat("normal", SEED, 53, (N, cout, D, H, W)), dtype, (0, 0), 3, D + 6)
    dwo, dbo = orc.conv3d_bwd_filter(xo, go, None, act=orc.ACT_NONE)
    dw = torch.zeros((cout, cin, 3, 3, 3), device="cuda")
    db = torch.zeros((cout,), device="cuda")
    for p0, p1 in [(1, D - 1), (0, 1), (D - 1, D)]:
        dwp, dbp = torch.empty_like(dw), torch.empty_like(db)
        h3d.conv3d_bwd_filter(xg.planes(p0, p1, 1, 1), gg.planes(p0, p1), None, dwp, dbp, h3d.ACT_NONE, 0.0)
        dw += dwp
        db += dbp
    tol_w = 1e-5 if dtype == "f32" else 2e-4
    close(from_dev(dw), dwo, tol_w)
    close(from_dev(db), dbo, tol_w)


# (N, Cin, Cout, D, H, W, halo, d_offset, d_global): fp32 tensors on the matrix cores.  Both instances of the forward kernel
# (one and two blocks of 16 output channels per workgroup; 2-row tiles since these volumes are small), channel counts that fill neither the groups of 4 input
# channels nor the blocks of 16 output channels, two workgroups of output channels, W beyond one 32-column tile with a
# ragged tail, W not a multiple of 4 (no 16-byte stores), H beyond one 8-row tile, more planes than one workgroup's four,
# boundary and interior shards, and backward-filter chunks of several tiles
F32_SHAPES = [
    (1, 6, 16, 5, 11, 44, 0, 0, 5),
    (2, 5, 20, 3, 9, 37, 1, 0, 3),
    (1, 40, 48, 6, 20, 40, 1, 6, 18),
    (2, 40, 48, 6, 20, 40, 1, 12, 18),
    (1, 18, 70, 2, 8, 66, 0, 0, 2),
    (1, 33, 7, 9, 4, 16, 1, 0, 12),
    (2, 8, 40, 16, 100, 132, 0, 0, 16),     # enough 8-row tiles to fill the chip: the 8-row instances
    (2, 36, 12, 16, 100, 132, 0, 0, 16),
    # at most 4 channels on the output side of the correlation (thin form: the three kh taps share a product) or on the
    # input side of backward-filter (the three kw taps share a product)
    (1, 4, 16, 6, 20, 40, 1, 0, 6),
    (2, 20, 3, 5, 9, 37, 0, 0, 5),
    (2, 1, 2, 3, 10, 72, 1, 3, 9),
    (2, 16, 4, 16, 100, 132, 0, 0, 16),
    # volumes at most 16 voxels wide: 16-column tiles (forward / BD) and 8-row x 16-column tiles (BF)
    (2, 20, 24, 4, 12, 8, 1, 0, 4),
    (1, 3, 6, 5, 9, 12, 0, 0, 5),
    (4, 5, 6, 16, 256, 16, 0, 0, 16),
]


kernels_seen = set()


@pytest.mark.parametrize("shape", F32_SHAPES)
def test_conv3d_fp32_matrix_core_kernels(shape):
    """Sec. III-C FP / BD / BF in the paper's own precision (fp32 storage and arithmetic) against the fp64 oracle at the
    1e-5 bar, with the kernel that ran checked by name."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W, halo, off, Dg = shape
    alpha = 0.01
    w, bias = _weights(Ci, Co, "f32", 60)
    wd, bd = to_dev(w, "f32"), to_dev(bias, "f32")
    hl = (halo, halo)
    xs = synth.flat("normal", SEED, 61, (N, Ci, D + 2 * halo, H, W))
    dzs = synth.flat("normal", SEED, 62, (N, Co, D + 2 * halo, H, W))
    for pl in range(D + 2 * halo):                    # canaries in halo planes outside the volume: never read
        g = off - halo + pl
        if g < 0 or g >= Dg:
            xs[:, :, pl] = 999.0
            dzs[:, :, pl] = 999.0
    xo, xg = slab_pair(xs, "f32", hl, off, Dg)
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=alpha)
    zg = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, "f32"), h3d.ACT_LEAKY, alpha)
    form = lambda c: "thin" if c <= 4 else ("1" if c <= 16 else "2")
    assert h3d.h3d_last_kernel().startswith("conv3d_f32_mfma_kernel<%s," % form(Co)), h3d.h3d_last_kernel()
    kernels_seen.add(h3d.h3d_last_kernel())
    close(from_dev(zg.t), zo.a, 1e-5)
    # backward passes: z and dz with the same halo (what the neighbours would have sent)
    zfull = synth.flat("normal", SEED, 63, (N, Co, D + 2 * halo, H, W))
    zso, zsg = slab_pair(zfull, "f32", hl, off, Dg)
    dzo, dzg = slab_pair(dzs, "f32", hl, off, Dg)
    dxo = orc.conv3d_bwd_data(dzo, zso, w, act=orc.ACT_LEAKY, alpha=alpha)
    dxg = h3d.conv3d_bwd_data(dzg, zsg, wd, dev_like(dxo, "f32"), h3d.ACT_LEAKY, alpha)
    assert h3d.h3d_last_kernel().startswith("conv3d_f32_mfma_kernel<%s," % form(Ci)), h3d.h3d_last_kernel()
    kernels_seen.add(h3d.h3d_last_kernel())
    close(from_dev(dxg.t), dxo.a, 1e-5)
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, zso, act=orc.ACT_LEAKY, alpha=alpha)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, zsg, dw, db, h3d.ACT_LEAKY, alpha)
    assert h3d.h3d_last_kernel() == ("bwd_filter_f32_mfma_kernel<thin>" if Ci <= 4 else "bwd_filter_f32_mfma_kernel"), h3d.h3d_last_kernel()
    close(from_dev(dw), dwo, 1e-5)
    close(from_dev(db), dbo, 1e-5)
    dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
    h3d.conv3d_bwd_filter(xg, dzg, zsg, dw2, db2, h3d.ACT_LEAKY, alpha)
    assert torch.equal(dw, dw2) and torch.equal(db, db2)
    # no activation, no saved output, no bias gradient wanted
    dwo_n, _ = orc.conv3d_bwd_filter(xo, dzo, None, act=orc.ACT_NONE)
    h3d.conv3d_bwd_filter(xg, dzg, None, dw2, None, h3d.ACT_NONE, 0.0)
    close(from_dev(dw2), dwo_n, 1e-5)


def _f32_random_shapes(k=12):
    rng = np.random.default_rng(SEED + 99)
    out = []
    for _ in range(k):
        ci = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 17, 24, 33]))
        co = int(rng.choice([1, 3, 4, 5, 9, 16, 17, 20, 32, 35]))
        d, halo = int(rng.integers(1, 8)), int(rng.integers(0, 2))
        out.append((int(rng.integers(1, 3)), ci, co, d, int(rng.integers(1, 23)), int(rng.choice([3, 8, 12, 16, 17, 31, 32, 40, 66])), halo,
                    int(rng.choice([0, 4])) if halo else 0))
    return out


@pytest.mark.parametrize("shape", _f32_random_shapes())
def test_conv3d_fp32_random_shapes(shape):
    """Seeded random shapes for the fp32 matrix-core kernels: channel counts on either side of the thin / one-block /
    two-block forms, widths on either side of the 16-column tiles, ragged rows, planes and halos in combinations nobody
    picked by hand; all three passes with the fused activation derivative, against the oracle at the fp32 bar."""
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W, halo, off = shape
    Dg = off + D + (4 if halo else 0)
    alpha = 0.01
    w, bias = _weights(Ci, Co, "f32", 70)
    wd, bd = to_dev(w, "f32"), to_dev(bias, "f32")
    hl = (halo, halo)
    xo, xg = slab_pair(synth.flat("normal", SEED, 71, (N, Ci, D + 2 * halo, H, W)), "f32", hl, off, Dg)
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=alpha)
    zg = h3d.conv3d_fwd(xg, wd, bd, dev_like(zo, "f32"), h3d.ACT_LEAKY, alpha)
    assert h3d.h3d_last_kernel().startswith("conv3d_f32_mfma_kernel"), h3d.h3d_last_kernel()
    close(from_dev(zg.t), zo.a, 1e-5, f"fwd {shape}")
    zso, zsg = slab_pair(synth.flat("normal", SEED, 73, (N, Co, D + 2 * halo, H, W)), "f32", hl, off, Dg)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, 72, (N, Co, D + 2 * halo, H, W)), "f32", hl, off, Dg)
    dxo = orc.conv3d_bwd_data(dzo, zso, w, act=orc.ACT_LEAKY, alpha=alpha)
    dxg = h3d.conv3d_bwd_data(dzg, zsg, wd, dev_like(dxo, "f32"), h3d.ACT_LEAKY, alpha)
    close(from_dev(dxg.t), dxo.a, 1e-5, f"bwd_data {shape}")
    dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, zso, act=orc.ACT_LEAKY, alpha=alpha)
    dw = torch.full((Co, Ci, 3, 3, 3), 777.0, device="cuda")
    db = torch.full((Co,), 777.0, device="cuda")
    h3d.conv3d_bwd_filter(xg, dzg, zsg, dw, db, h3d.ACT_LEAKY, alpha)
    assert h3d.h3d_last_kernel().startswith("bwd_filter_f32_mfma_kernel"), h3d.h3d_last_kernel()
    close(from_dev(dw), dwo, 1e-5, f"dw {shape}")
    close(from_dev(db), dbo, 1e-5, f"db {shape}")


def test_conv3d_fp32_every_instance_was_run():
    """The shapes above reach the instances of the fp32 forward / backward-data kernel (channel-block form x tile rows x
    tile halves) (collected from the library's
    own report of the kernel it ran); skipped when that test was not run in this process."""
    if not kernels_seen:
        pytest.skip("test_conv3d_fp32_matrix_core_kernels did not run in this process")
    want = {"conv3d_f32_mfma_kernel<%s,%d,2>" % (cb, tr) for cb in ("1", "2", "thin") for tr in (2, 8)}
    want |= {"conv3d_f32_mfma_kernel<%s,1>" % k for k in ("1,8", "1,2", "2,2", "thin,2")}
    assert want <= kernels_seen, (want - kernels_seen, kernels_seen)


def test_plane_run_views_are_rejected_elsewhere():
    import paper_2007_12856_amd as h3d
    _, xg = slab_pair(synth.flat("normal", SEED, 54, (1, 2, 6, 4, 8)), "bf16")
    _, yg = slab_pair(np.zeros((1, 2, 3, 2, 4)), "bf16")
    import torch
    buf = torch.empty(2 * 2 * 4 * 8, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(h3d.H3DError) as e:
        h3d.halo_pack(xg.planes(0, 4), h3d.FACE_D_LO, 1, buf)
    assert e.value.status == -2
    with pytest.raises(h3d.H3DError) as e:
        x4 = h3d.Slab(torch.zeros((2, 4, 6, 4, 8), dtype=torch.bfloat16, device="cuda"))      # (one sample: its first channels are packed memory)
        h3d.concat_c(x4.channels(0, 2), x4.channels(2, 4), h3d.Slab(torch.empty_like(x4.t)))
    assert e.value.status == -2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_halo_recompute_two_stacked_convs(dtype):
    """A 2-plane halo serves two stacked convolutions (U-Net-shaped level): the first also produces
    its output's halo plane; beyond the global boundary that plane must be zero, not act(bias)."""
    import paper_2007_12856_amd as h3d
    Ci, Cm, Co, Dg, H, W, d = 1, 8, 16, 8, 12, 20, 4
    wa, ba = _weights(Ci, Cm, dtype, 40)
    wb, bb = _weights(Cm, Co, dtype, 42)
    for off in (0, 4):
        xs = cut("normal", SEED, 7, (1, Ci, Dg, H, W), off, d, (2, 2))
        xo, xg = slab_pair(xs, dtype, (2, 2), off, Dg)
        ao = orc.conv3d_fwd(xo, wa, ba, cout_halo=(1, 1), act=orc.ACT_RELU)
        ag = h3d.conv3d_fwd(xg, to_dev(wa, dtype), to_dev(ba, "f32"), dev_like(ao, dtype), h3d.ACT_RELU, 0.0)
        close(from_dev(ag.t), ao.a, TOL[dtype])
        outside = 0 if off == 0 else -1
        assert not from_dev(ag.t)[:, :, outside].any()
        aqo, aqg = slab_pair(ao.a, dtype, (1, 1), off, Dg)
        bo = orc.conv3d_fwd(aqo, wb, bb, act=orc.ACT_RELU)
        bg = h3d.conv3d_fwd(aqg, to_dev(wb, dtype), to_dev(bb, "f32"), dev_like(bo, dtype), h3d.ACT_RELU, 0.0)
        close(from_dev(bg.t), bo.a, TOL[dtype])


def test_error_paths_do_not_launch():
    import torch
    import paper_2007_12856_amd as h3d
    x = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda"), 0, 0, 4, 16)      # interior shard without halo
    z = x.like(3)
    w = torch.zeros((3, 2, 3, 3, 3), device="cuda")
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_fwd(x, w, None, z)
    assert e.value.status == -4
    zbad = h3d.Slab(torch.zeros((1, 3, 4, 4, 5), device="cuda"), 0, 0, 4, 16)
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_fwd(x, w, None, zbad)
    assert e.value.status == -1
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_fwd(h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda")), w, None,
                       h3d.Slab(torch.zeros((1, 3, 4, 4, 4), device="cuda")), act=7)
    assert e.value.status == -1
    # workspace too small is reported, not overrun
    import ctypes
    xd, zd = h3d.Slab(torch.zeros((1, 2, 4, 4, 4), device="cuda")), h3d.Slab(torch.zeros((1, 3, 4, 4, 4), device="cuda"))
    st = h3d.lib().h3d_conv3d_fwd(h3d.handle(), ctypes.byref(xd.desc()), ctypes.c_void_p(w.data_ptr()), None,
                                  ctypes.byref(zd.desc()), 0, 0.0, None, 0, None)
    assert st == -3


def test_empty_shard():
    import torch
    import paper_2007_12856_amd as h3d
    x = h3d.Slab(torch.zeros((0, 2, 4, 4, 4), device="cuda"))
    z = h3d.Slab(torch.zeros((0, 3, 4, 4, 4), device="cuda"))
    w = torch.ones((3, 2, 3, 3, 3), device="cuda")
    h3d.conv3d_fwd(x, w, None, z)
    dw = torch.full((3, 2, 3, 3, 3), 5.0, device="cuda")
    db = torch.full((3,), 5.0, device="cuda")
    h3d.conv3d_bwd_filter(x, z, None, dw, db)
    torch.cuda.synchronize()
    assert not dw.any() and not db.any()
