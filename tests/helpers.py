"""Shared plumbing for the GPU parity tests: build the same slab twice — once as fp64 for the
oracle, once as a device tensor for the HIP path — from one seeded array rounded to the storage type."""
from __future__ import annotations

import numpy as np

import oracle as orc
import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative L2 bars of the benchmark spec


def quantize(a, dtype: str) -> np.ndarray:
    """Values after one rounding to the storage type, as float64."""
    return (synth.round_f32(a) if dtype == "f32" else synth.round_bf16(a)).astype(np.float64)


def to_dev(a, dtype: str):
    import torch
    a = np.ascontiguousarray(a)
    if dtype == "f32":
        return torch.from_numpy(a.astype(np.float32)).cuda()
    bits = synth.f32_to_bf16_bits(a.astype(np.float32))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_dev(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_l2(got, ref) -> float:
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return float(num / den) if den > 0 else float(num)


def slab_pair(a, dtype: str, halo=(0, 0), d_offset=0, d_global=None):
    """(oracle Slab, device Slab) holding identical values; `a` is [N,C,stored planes,H,W]."""
    import paper_2007_12856_amd as h3d
    q = quantize(a, dtype)
    o = orc.Slab(q, halo[0], halo[1], d_offset, d_global)
    g = h3d.Slab(to_dev(q, dtype), halo[0], halo[1], d_offset, o.d_global)
    return o, g


def dev_like(o: orc.Slab, dtype: str, fill=None):
    """A device slab with the geometry of oracle slab `o` (filled with a canary unless told otherwise)."""
    import torch
    import paper_2007_12856_amd as h3d
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    t = torch.full(o.a.shape, 12345.0 if fill is None else fill, dtype=td, device="cuda")
    return h3d.Slab(t, o.halo_lo, o.halo_hi, o.d_offset, o.d_global)


def cut(kind, seed, stream, full_shape, off, d, halo, lo=-1.0, hi=1.0):
    """Stored planes [off-halo_lo, off+d+halo_hi) of the seeded virtual volume (zeros outside it)."""
    return synth.slab(kind, seed, stream, full_shape, off - halo[0], off + d + halo[1], lo, hi)
