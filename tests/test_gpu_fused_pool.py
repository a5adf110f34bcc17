"""GPU parity of the convolution forward fused with the average pooling after it, the sign mask, and the pooling
backward that reads the mask instead of the saved output."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import TOL, dev_like, from_dev, quantize, close, rel_l2, slab_pair, to_dev

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED + 7


def _weights(cin, cout, dtype, stream):
    b = np.sqrt(3.0 / (27 * cin))
    w = quantize(synth.flat("uniform", SEED, stream, (cout, cin, 3, 3, 3), -b, b), dtype)
    bias = synth.round_f32(synth.flat("uniform", SEED, stream + 1, (cout,), -0.1, 0.1)).astype(np.float64)
    return w, bias


def _mask_from_stored(z_stored: np.ndarray) -> np.ndarray:
    out = np.zeros(z_stored.shape[:4] + (z_stored.shape[4] // 8,), dtype=np.uint8)
    for k in range(8):
        out |= (z_stored[..., k::8] > 0).astype(np.uint8) << k
    return out


# (N, Cin, Cout, D, H, W, x halo): fused kernel shapes (Cin <= 4, Cout <= 32, even D and H, W a multiple of 8: one and
# several tiles in every direction, ragged last tiles, two row blocks of output channels), then shapes that take
# the three-pass route (more input channels; odd multiple of 8 is fine, W = 12 is not a multiple of 8: no mask)
FUSED = [(1, 4, 16, 4, 4, 64, 0), (2, 4, 16, 6, 10, 72, 0), (1, 1, 32, 8, 6, 136, 0), (1, 3, 20, 2, 2, 8, 0),
         (1, 4, 16, 4, 8, 64, 1),
         # at most 16 output channels and at least 8 rows: the row-streaming kernel (several row segments, ragged plane
         # quads, one and two column tiles, fewer than 4 input channels)
         (1, 4, 16, 8, 20, 136, 0), (2, 3, 12, 6, 8, 128, 0), (1, 2, 5, 2, 16, 8, 0), (1, 4, 16, 4, 64, 256, 0)]
UNFUSED = [(1, 8, 16, 4, 6, 16, 0), (1, 16, 8, 2, 4, 40, 0)]


@pytest.mark.parametrize("store_z", [True, False])
@pytest.mark.parametrize("shape", FUSED + UNFUSED)
def test_conv_fwd_pool_matches_oracle_composition(shape, store_z):
    import torch
    import paper_2007_12856_amd as h3d
    N, Ci, Co, D, H, W, halo = shape
    dtype = "bf16"
    Dg, off = (D + 4, 2) if halo else (D, 0)          # the shard starts at an even plane: no window straddles a face
    w, bias = _weights(Ci, Co, dtype, 10)
    xo, xg = slab_pair(synth.flat("normal", SEED, 1, (N, Ci, D + 2 * halo, H, W)), dtype, (halo, halo), off, Dg)
    zo = orc.conv3d_fwd(xo, w, bias, act=orc.ACT_LEAKY, alpha=0.01)
    zq = orc.Slab(quantize(zo.a, dtype), 0, 0, zo.d_offset, zo.d_global)       # the pooling reads the stored activation
    yo = orc.pool3d_fwd(zq, orc.POOL_AVG)
    zg = dev_like(zo, dtype)
    yg = dev_like(yo, dtype)
    fused = shape in FUSED
    mask = torch.full((h3d.act_mask_bytes(xg, zg),), 0xAA, dtype=torch.uint8, device="cuda")
    if not store_z and not fused:
        with pytest.raises(h3d.H3DError) as e:
            h3d.conv3d_fwd_pool(xg, to_dev(w, dtype), to_dev(bias, "f32"), (N, Co, D, H, W), yg, None, h3d.ACT_LEAKY, 0.01)
        assert e.value.status == -2
        return
    h3d.conv3d_fwd_pool(xg, to_dev(w, dtype), to_dev(bias, "f32"), zg if store_z else (N, Co, D, H, W), yg, mask, h3d.ACT_LEAKY, 0.01)
    close(from_dev(yg.t), yo.a, 4e-3)
    if store_z:
        z_gpu = from_dev(zg.t)
        close(z_gpu, zo.a, TOL[dtype])
        # the mask is the sign of what the GPU itself stored, bit for bit
        assert np.array_equal(mask.cpu().numpy().reshape(N, Co, D, H, W // 8), _mask_from_stored(z_gpu))
    else:
        # without z: compare against the oracle's mask, except where the activation is within rounding of zero
        got = mask.cpu().numpy().reshape(N, Co, D, H, W // 8)
        want = orc.act_mask(zq)
        diff = np.unpackbits((got ^ want)[..., None], axis=-1, bitorder="little").reshape(N, Co, D, H, W).astype(bool)
        assert np.all(np.abs(zo.a[diff]) <= 1e-2 * np.abs(zo.a).max())
        assert diff.mean() < 1e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_act_mask_kernel_is_bit_exact(dtype):
    import torch
    import paper_2007_12856_amd as h3d
    a = synth.flat("normal", SEED, 3, (2, 3, 6, 5, 24))
    a[0, 1, 2] = 0.0                                   # zeros are not positive
    zo, zg = slab_pair(a, dtype, (1, 1), 4, 12)
    mask = torch.zeros((h3d.act_mask_bytes(zg, zg),), dtype=torch.uint8, device="cuda")
    h3d.act_mask(zg, mask)
    assert np.array_equal(mask.cpu().numpy().reshape(2, 3, 4, 5, 3), orc.act_mask(zo))


@pytest.mark.parametrize("shape,halo", [((2, 3, 4, 6, 32), (0, 0)), ((1, 5, 2, 4, 80), (1, 1)), ((1, 16, 8, 32, 64), (1, 0))])
@pytest.mark.parametrize("act", ["relu", "leaky"])
def test_pool_bwd_from_mask_equals_pool_bwd_from_saved_output(shape, halo, act):
    """Same bits as the pass that reads z itself, and parity with the oracle's pooling backward times the derivative."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    code, alpha = (h3d.ACT_RELU, 0.0) if act == "relu" else (h3d.ACT_LEAKY, 0.01)
    za = synth.flat("normal", SEED, 5, (N, C, halo[0] + d + halo[1], H, W))
    za[:, :, :, 0] = 0.0
    zo, zg = slab_pair(za, "bf16", halo, 4, 4 + d + 6)
    dyo, dyg = slab_pair(synth.flat("normal", SEED, 6, (N, C, d // 2, H // 2, W // 2)), "bf16", (0, 0), 2, (4 + d + 6) // 2)
    mask = torch.zeros((h3d.act_mask_bytes(zg, zg),), dtype=torch.uint8, device="cuda")
    h3d.act_mask(zg, mask)
    g1 = h3d.Slab(torch.full(za.shape, 7.0, dtype=torch.bfloat16, device="cuda"), halo[0], halo[1], 4, 4 + d + 6)
    g2 = h3d.Slab(torch.full(za.shape, 7.0, dtype=torch.bfloat16, device="cuda"), halo[0], halo[1], 4, 4 + d + 6)
    h3d.pool3d_bwd_act(dyg, None, zg, g1, h3d.POOL_AVG, code, alpha)
    h3d.pool3d_bwd_mask(dyg, mask, g2, code, alpha)
    assert torch.equal(g1.t, g2.t)
    dxo = orc.pool3d_bwd(dyo, zo, orc.POOL_AVG, dx_halo=halo)
    want = dxo.interior * np.where(zo.interior > 0, 1.0, alpha)
    close(from_dev(g2.interior), want, 4e-3)


@pytest.mark.parametrize("shape,halo", [((2, 3, 4, 6, 32), (0, 0)), ((1, 5, 2, 4, 80), (1, 1)), ((1, 16, 8, 32, 64), (1, 0))])
def test_pool_fwd_with_mask_equals_the_two_separate_passes(shape, halo):
    """The pooling forward that also writes the sign mask of its input: the pooled tensor of pool3d_fwd and the mask of
    act_mask, bit for bit; halo planes of the input are not touched, halo planes of the output stay as they were."""
    import torch
    import paper_2007_12856_amd as h3d
    N, C, d, H, W = shape
    za = synth.flat("normal", SEED, 15, (N, C, halo[0] + d + halo[1], H, W))
    za[:, :, :, 1] = 0.0
    _, zg = slab_pair(za, "bf16", halo, 4, 4 + d + 6)
    mk = lambda: h3d.Slab(torch.full((N, C, d // 2 + 2, H // 2, W // 2), 9.0, dtype=torch.bfloat16, device="cuda"), 1, 1, 2, (4 + d + 6) // 2)
    y1, y2 = mk(), mk()
    m1 = torch.zeros((h3d.act_mask_bytes(zg, zg),), dtype=torch.uint8, device="cuda")
    m2 = torch.full_like(m1, 0xAA)
    h3d.pool3d_fwd(zg, y1, h3d.POOL_AVG)
    h3d.act_mask(zg, m1)
    h3d.pool3d_fwd_mask(zg, y2, m2)
    assert torch.equal(y1.t, y2.t) and torch.equal(m1, m2)
    with pytest.raises(h3d.H3DError) as e:                      # w not a multiple of 16
        zz = h3d.Slab(torch.zeros((1, 1, 2, 2, 8), dtype=torch.bfloat16, device="cuda"))
        h3d.pool3d_fwd_mask(zz, h3d.Slab(torch.zeros((1, 1, 1, 1, 4), dtype=torch.bfloat16, device="cuda")), m2)
    assert e.value.status == -2
