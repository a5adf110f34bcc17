"""Seeded synthetic inputs for the 3-D convolution hot path.

This module only *draws numbers*.  It holds none of the arithmetic of the
method (no convolution, pooling, activation or halo logic) and is the one
module that both the CPU oracle's tests and the HIP path's tests/bench use,
so the two sides see identical bytes.

Every value is a pure function of (seed, stream, global linear index of the
element in the UNSHARDED N,C,D,H,W tensor).  A depth slab with halo planes is
therefore cut from the same virtual full volume without materialising it, and
planes that fall outside the global volume come back as zero ("same" padding
of the network table in Sec. IV: all layers use zero padding).

Value recipes stand in for the data the paper trains on (Sec. II-C): the
CosmoFlow cubes are non-negative, sparse, heavy-tailed particle counts, drawn
here as log(1+k) with k a Poisson count whose rate is log-normal; the CT
volumes of the 3D U-Net are stood in for by unit normals.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 200712856

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function (public-domain finaliser), vectorised."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _C1
    z ^= z >> np.uint64(27)
    z *= _C2
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, stream: int) -> np.uint64:
    k = (int(seed) * 0x9E3779B97F4A7C15 + int(stream) * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF
    return _mix64(np.array([k], dtype=np.uint64))[0]


def u01(seed: int, stream: int, idx: np.ndarray) -> np.ndarray:
    """Uniform doubles in the open interval (0,1), one per counter in `idx`."""
    with np.errstate(over="ignore"):
        bits = _mix64((idx.astype(np.uint64) + np.uint64(1)) * _GOLD ^ _key(seed, stream))
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _transform(kind: str, seed: int, stream: int, idx: np.ndarray, lo: float, hi: float) -> np.ndarray:
    if kind == "uniform":
        return lo + (hi - lo) * u01(seed, stream, idx)
    if kind == "normal":
        u1 = u01(seed, 2 * stream + 1000003, idx)
        u2 = u01(seed, 2 * stream + 1000004, idx)
        return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    if kind == "cosmo":
        # log(1+k), k ~ Poisson(exp(g)), g ~ N(0,1) clipped to [-3,3]; Poisson by
        # sequential inversion of one uniform (active set shrinks every term).
        g = np.clip(_transform("normal", seed, stream, idx, 0.0, 0.0), -3.0, 3.0)
        lam = np.exp(g)
        u = u01(seed, 2 * stream + 2000003, idx)
        k = np.zeros(idx.shape, dtype=np.int64)
        p = np.exp(-lam)
        cdf = p.copy()
        active = np.nonzero(u > cdf)[0]
        kk = 0
        while active.size and kk < 200:
            kk += 1
            p[active] *= lam[active] / kk
            cdf[active] += p[active]
            k[active] = kk
            active = active[u[active] > cdf[active]]
        return np.log1p(k.astype(np.float64))
    raise ValueError(f"unknown kind {kind!r}")


def flat(kind: str, seed: int, stream: int, shape, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """A packed tensor of `shape` (weights, biases, targets, unsharded activations)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = _transform(kind, seed, stream, np.arange(s, e, dtype=np.uint64), lo, hi)
    return out.reshape(shape)


def slab(kind: str, seed: int, stream: int, full_shape, p_lo: int, p_hi: int,
         lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """Global depth planes [p_lo, p_hi) of the virtual N,C,D,H,W tensor `full_shape`.

    Returns float64 [N, C, p_hi - p_lo, H, W].  Planes outside [0, D) are zero.
    """
    N, C, D, H, W = (int(v) for v in full_shape)
    out = np.zeros((N, C, p_hi - p_lo, H, W), dtype=np.float64)
    a, b = max(p_lo, 0), min(p_hi, D)
    if b <= a:
        return out
    plane = H * W
    # chunk so temporaries stay below ~32 Mi elements
    dstep = max(1, (1 << 22) // plane)
    for n in range(N):
        for c in range(C):
            base = (n * C + c) * D
            for d0 in range(a, b, dstep):
                d1 = min(b, d0 + dstep)
                idx = np.arange((base + d0) * plane, (base + d1) * plane, dtype=np.uint64)
                out[n, c, d0 - p_lo:d1 - p_lo] = _transform(kind, seed, stream, idx, lo, hi).reshape(d1 - d0, H, W)
    return out


# ---------------------------------------------------------------------------
# storage-type rounding (plumbing shared by both sides: inputs are rounded to
# the storage type ONCE, before either implementation sees them)
# ---------------------------------------------------------------------------

def round_f32(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float64).astype(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + rnd) >> np.uint32(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Value of `a` after one RNE rounding to bf16, as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, dtype=np.float64).astype(np.float32)))
