"""The backward-filter entry point that takes no workspace and allocates nothing (for callers under graph capture or in
loops that may not call hipMalloc): same bits as h3d_conv3d_bwd_filter, on two calls in a row that share the library's
scratch array, the second on a smaller input; shapes beyond the array are refused before any launch."""
import numpy as np
import pytest

import oracle as orc
import synth
from helpers import close, from_dev, slab_pair

pytestmark = pytest.mark.gpu
SEED = synth.BASE_SEED + 31


def _case(N, Ci, Co, D, H, W, stream):
    Dg, off = D + 2, 1
    xo, xg = slab_pair(synth.flat("normal", SEED, stream, (N, Ci, D + 2, H, W)), "bf16", (1, 1), off, Dg)
    dzo, dzg = slab_pair(synth.flat("normal", SEED, stream + 1, (N, Co, D, H, W)), "bf16", (0, 0), off, Dg)
    return xo, xg, dzo, dzg


def test_static_scratch_backward_filter_matches_the_workspace_call_twice_in_a_row(monkeypatch):
    import torch
    import paper_2007_12856_amd as h3d
    monkeypatch.setenv("H3D_BF_ROW32", "1")     # the first shape then takes the many-channel kernel (test hook of the library)
    assert h3d.static_scratch_bytes() == 96 << 20
    # first a call that fills a large part of the array, then a smaller one whose partial sums overlay its leftovers
    for k, shape in enumerate([(2, 64, 64, 6, 40, 64), (2, 32, 64, 4, 40, 64), (1, 4, 16, 4, 32, 64), (1, 16, 8, 2, 9, 20)]):
        N, Ci, Co, D, H, W = shape
        xo, xg, dzo, dzg = _case(*shape, stream=10 * k)
        dw_ws = torch.full((Co, Ci, 3, 3, 3), 5.0, device="cuda")
        db_ws = torch.full((Co,), 5.0, device="cuda")
        h3d.conv3d_bwd_filter(xg, dzg, None, dw_ws, db_ws, h3d.ACT_NONE, 0.0)
        dw, db = torch.full_like(dw_ws, -7.0), torch.full_like(db_ws, -7.0)
        torch.cuda.synchronize()
        allocs = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]      # allocations so far (never decreases)
        before = allocs()
        h3d.conv3d_bwd_filter_static(xg, dzg, None, dw, db, h3d.ACT_NONE, 0.0)
        torch.cuda.synchronize()
        assert allocs() == before                          # the binding asked torch for nothing either
        assert torch.equal(dw, dw_ws) and torch.equal(db, db_ws), shape          # same kernels, same order: same bits
        dwo, dbo = orc.conv3d_bwd_filter(xo, dzo, None, act=orc.ACT_NONE)
        close(from_dev(dw), dwo, 2e-4, f"dw {shape}")
        close(from_dev(db), dbo, 2e-4, f"db {shape}")


def test_static_scratch_refuses_shapes_beyond_the_array():
    import torch
    import paper_2007_12856_amd as h3d
    # 1024 -> 1024 channels: 113 MB of partial sums per chunk of voxels
    x = h3d.Slab(torch.zeros((1, 1024, 2, 8, 32), dtype=torch.bfloat16, device="cuda"))
    dz = h3d.Slab(torch.zeros((1, 1024, 2, 8, 32), dtype=torch.bfloat16, device="cuda"))
    need = h3d.h3d_conv3d_workspace_bytes(h3d.OP_BWD_FILTER, x, dz)
    assert need > h3d.static_scratch_bytes()
    dw = torch.full((1024, 1024, 3, 3, 3), 3.0, device="cuda")
    with pytest.raises(h3d.H3DError) as e:
        h3d.conv3d_bwd_filter_static(x, dz, None, dw, None, h3d.ACT_NONE, 0.0)
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert bool((dw == 3.0).all())          # nothing was launched
