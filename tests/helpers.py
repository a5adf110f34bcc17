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


def elem_bound(tol: float) -> float:
    """Per-element factor e that goes with a relative-L2 bar: 2^-7 for the bf16 bar of 2e-2 (one bf16 ulp is at most 2^-7
    of the value: an element may be off by its own rounding plus a little accumulated error, never by a whole voxel's
    worth), the bar itself below that (fp32 results: 1e-5; fp32 sums of bf16 products: 2e-4; pooled bf16 values: 4e-3)."""
    return tol if tol < 2e-2 else 2.0 ** -7 * (tol / 2e-2)


# Backward-filter with the activation derivative fused, bf16 tensors: g = dz * act'(z) is rounded to bf16 ONCE before the
# matrix cores read it (the oracle keeps the product in fp64).  A filter gradient that is a single product (one-voxel
# volumes) or a sum of few carries that rounding whole: half a bf16 ulp = 2^-8 of the element.  Unmasked calls multiply
# bf16 inputs exactly and stay on the fp32-sum bar.
def elem_masked_bf(dtype: str):
    return None if dtype == "f32" else 2.0 ** -8


def close(got, ref, tol: float, what: str = "", elem: float | None = None, outliers: float = 0.0) -> bool:
    """The two parity checks every GPU-vs-oracle comparison makes:
    (1) relative L2 over the whole tensor <= tol (the bar of the benchmark spec), and
    (2) element by element: |got - ref| <= e |ref| + e rms(ref), with e = elem_bound(tol) unless given.  The rms term is
        the floor for elements near zero (a sum of many products cancels to any small value; its error does not).
    `outliers`: fraction of elements that may exceed (2) (0 except where the two sides legitimately take a decision from
    their own data, e.g. the sign of an activation within rounding of zero, stated at the call)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    r = rel_l2(got, ref)
    assert r <= tol, f"{what}: rel-L2 {r:.3e} > {tol:.1e}"
    e = elem_bound(tol) if elem is None else elem
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bad = np.abs(got - ref) > e * np.abs(ref) + e * rms
    frac = float(bad.mean()) if bad.size else 0.0
    if frac > outliers:
        idx = np.unravel_index(int(np.argmax(np.abs(got - ref) - e * np.abs(ref))), ref.shape) if ref.ndim else ()
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements ({frac:.2e} > {outliers:.1e}) outside "
                             f"|d| <= {e:.2e} (|ref| + rms {rms:.3e}); worst at {idx}: got {got[idx]!r} ref {ref[idx]!r}")
    return True


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
