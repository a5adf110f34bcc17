"""CPU fp64 oracle — TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct implementations of what the hot path computes
(paper Sec. III-A layer computations on a depth slab; Sec. III-C passes FP/BD/BF).
The arithmetic lives in `h3d_oracle.c` (direct loop nests, fp64) and, for the
index-only and library-primitive steps, in numpy below.  Nothing here imports
or is imported by the HIP package; only tests, the smoke check and the bench's
CPU-baseline leg may use it.

Pins (tests/test_oracle_*.py): brute force against an independently written
definition, a library cross-check (torch CPU float64 + autograd), the
delta-input identity, closed forms for constant inputs, linearity, the adjoint
identity, finite differences, bit-exact shard consistency, the conv-FLOP and
parameter counts printed in Table I.  Unpinned by the paper itself: every
numeric layer output (the paper prints no worked example).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libh3d_oracle.so")
_SRC = os.path.join(_HERE, "h3d_oracle.c")

ACT_NONE, ACT_RELU, ACT_LEAKY = 0, 1, 2
POOL_AVG, POOL_MAX = 0, 1
FACE_D_LO, FACE_D_HI = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


@dataclass
class Slab:
    """A depth slab of an N,C,D,H,W tensor; `a` is float64 [N, C, halo_lo+d+halo_hi, H, W]."""
    a: np.ndarray
    halo_lo: int = 0
    halo_hi: int = 0
    d_offset: int = 0
    d_global: int | None = None

    def __post_init__(self):
        self.a = np.ascontiguousarray(self.a, dtype=np.float64)
        assert self.a.ndim == 5
        if self.d_global is None:
            self.d_global = self.d
        assert self.d >= 0

    @property
    def d(self) -> int:
        return self.a.shape[2] - self.halo_lo - self.halo_hi

    @property
    def interior(self) -> np.ndarray:
        return self.a[:, :, self.halo_lo:self.halo_lo + self.d]

    def geom(self):
        n, c, _, h, w = self.a.shape
        return (ctypes.c_int64 * 9)(n, c, self.d, h, w, self.halo_lo, self.halo_hi, self.d_offset, self.d_global)

    def like(self, channels: int, halo_lo: int = 0, halo_hi: int = 0, fill: float = np.nan) -> "Slab":
        n, _, _, h, w = self.a.shape
        a = np.full((n, channels, halo_lo + self.d + halo_hi, h, w), fill, dtype=np.float64)
        return Slab(a, halo_lo, halo_hi, self.d_offset, self.d_global)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: status {rc}")


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def conv3d_fwd(x: Slab, w, bias, cout_halo=(0, 0), act=ACT_NONE, alpha=0.0) -> Slab:
    """z = act(b + w (*) x~), 3x3x3, stride 1, zero padding 1 (Table I caption; Sec. III-A)."""
    w = _f64(w)
    bias = _f64(bias)
    assert w.shape[1:] == (x.a.shape[1], 3, 3, 3)
    z = x.like(w.shape[0], cout_halo[0], cout_halo[1])
    _chk(_L().orc_conv3d_fwd(_p(x.a), x.geom(), _p(w), _p(bias), _p(z.a), z.geom(), int(act),
                             ctypes.c_double(alpha)), "conv3d_fwd")
    return z


def conv3d_bwd_data(dz: Slab, z: Slab | None, w, dx_halo=(0, 0), act=ACT_NONE, alpha=0.0) -> Slab:
    """BD pass (Sec. III-C): dx = sum_{co,k} w[co,ci,k] * (dz*act'(z))~[q-k+1]."""
    w = _f64(w)
    assert w.shape[0] == dz.a.shape[1] and w.shape[2:] == (3, 3, 3)
    dx = dz.like(w.shape[1], dx_halo[0], dx_halo[1])
    _chk(_L().orc_conv3d_bwd_data(_p(dz.a), dz.geom(), _p(z.a) if z is not None else None,
                                  z.geom() if z is not None else None, _p(w), _p(dx.a), dx.geom(), int(act),
                                  ctypes.c_double(alpha)), "conv3d_bwd_data")
    return dx


def conv3d_bwd_filter(x: Slab, dz: Slab, z: Slab | None, act=ACT_NONE, alpha=0.0):
    """BF pass (Sec. III-C): the shard's partial dw [cout,cin,3,3,3] and db [cout]."""
    cin, cout = x.a.shape[1], dz.a.shape[1]
    dw = np.zeros((cout, cin, 3, 3, 3), dtype=np.float64)
    db = np.zeros((cout,), dtype=np.float64)
    _chk(_L().orc_conv3d_bwd_filter(_p(x.a), x.geom(), _p(dz.a), dz.geom(), _p(z.a) if z is not None else None,
                                    z.geom() if z is not None else None, _p(dw), _p(db), int(act),
                                    ctypes.c_double(alpha)), "conv3d_bwd_filter")
    return dw, db


def convk_fwd(x: Slab, w, bias, act=ACT_NONE, alpha=0.0) -> Slab:
    """Odd filter edge K (5 for the 5x5x5 filters of Sec. III-A), stride 1, zero padding K//2; shard interior only."""
    w = _f64(w)
    bias = _f64(bias)
    k = w.shape[2]
    assert w.shape[1:] == (x.a.shape[1], k, k, k)
    z = x.like(w.shape[0])
    _chk(_L().orc_convk_fwd(k, _p(x.a), x.geom(), _p(w), _p(bias), _p(z.a), z.geom(), int(act),
                            ctypes.c_double(alpha)), "convk_fwd")
    return z


def convk_bwd_data(dz: Slab, z: Slab | None, w, act=ACT_NONE, alpha=0.0) -> Slab:
    """dx = sum_{co,k} w[co,ci,k] * (dz*act'(z))~[q-k+K//2] on the shard interior."""
    w = _f64(w)
    k = w.shape[2]
    assert w.shape[0] == dz.a.shape[1] and w.shape[2:] == (k, k, k)
    dx = dz.like(w.shape[1])
    _chk(_L().orc_convk_bwd_data(k, _p(dz.a), dz.geom(), _p(z.a) if z is not None else None,
                                 z.geom() if z is not None else None, _p(w), _p(dx.a), dx.geom(), int(act),
                                 ctypes.c_double(alpha)), "convk_bwd_data")
    return dx


def convk_bwd_filter(k: int, x: Slab, dz: Slab, z: Slab | None, act=ACT_NONE, alpha=0.0):
    """The shard's partial dw [cout,cin,k,k,k] and db [cout]."""
    cin, cout = x.a.shape[1], dz.a.shape[1]
    dw = np.zeros((cout, cin, k, k, k), dtype=np.float64)
    db = np.zeros((cout,), dtype=np.float64)
    _chk(_L().orc_convk_bwd_filter(k, _p(x.a), x.geom(), _p(dz.a), dz.geom(), _p(z.a) if z is not None else None,
                                   z.geom() if z is not None else None, _p(dw), _p(db), int(act),
                                   ctypes.c_double(alpha)), "convk_bwd_filter")
    return dw, db


def _s2_out(x: Slab, channels: int, halo_lo: int = 0, halo_hi: int = 0, fill: float = np.nan) -> Slab:
    n, _, _, h, w = x.a.shape
    a = np.full((n, channels, halo_lo + x.d // 2 + halo_hi, (h + 1) // 2, (w + 1) // 2), fill, dtype=np.float64)
    return Slab(a, halo_lo, halo_hi, x.d_offset // 2, x.d_global // 2)


def conv3d_s2_fwd(x: Slab, w, bias, act=ACT_NONE, alpha=0.0) -> Slab:
    """Stride-2 3x3x3 convolution (Table I, fourth convolution): y[p] = act(b + sum_k w[k] x~[2p+k-1])."""
    w = _f64(w)
    bias = _f64(bias)
    assert w.shape[1:] == (x.a.shape[1], 3, 3, 3)
    y = _s2_out(x, w.shape[0])
    _chk(_L().orc_conv3d_s2_fwd(_p(x.a), x.geom(), _p(w), _p(bias), _p(y.a), y.geom(), int(act),
                                ctypes.c_double(alpha)), "conv3d_s2_fwd")
    return y


def conv3d_s2_bwd_data(dy: Slab, y: Slab | None, w, x_like: Slab, act=ACT_NONE, alpha=0.0) -> Slab:
    """dx of the stride-2 convolution on the interior of the input shard described by `x_like`."""
    w = _f64(w)
    assert w.shape[0] == dy.a.shape[1] and w.shape[2:] == (3, 3, 3)
    dx = x_like.like(w.shape[1])
    _chk(_L().orc_conv3d_s2_bwd_data(_p(dy.a), dy.geom(), _p(y.a) if y is not None else None,
                                     y.geom() if y is not None else None, _p(w), _p(dx.a), dx.geom(), int(act),
                                     ctypes.c_double(alpha)), "conv3d_s2_bwd_data")
    return dx


def conv3d_s2_bwd_filter(x: Slab, dy: Slab, y: Slab | None, act=ACT_NONE, alpha=0.0):
    """The shard's partial dw [cout,cin,3,3,3] and db [cout] of the stride-2 convolution."""
    cin, cout = x.a.shape[1], dy.a.shape[1]
    dw = np.zeros((cout, cin, 3, 3, 3), dtype=np.float64)
    db = np.zeros((cout,), dtype=np.float64)
    _chk(_L().orc_conv3d_s2_bwd_filter(_p(x.a), x.geom(), _p(dy.a), dy.geom(), _p(y.a) if y is not None else None,
                                       y.geom() if y is not None else None, _p(dw), _p(db), int(act),
                                       ctypes.c_double(alpha)), "conv3d_s2_bwd_filter")
    return dw, db


def act_bwd(dz: Slab, dz2: Slab | None, z: Slab, act: int, alpha: float = 0.0, g_halo=(0, 0)) -> Slab:
    """g = (dz + dz2) * (z > 0 ? 1 : slope) on the interior (activation derivative, Sec. IV); halo planes of g are zero."""
    slope = alpha if act == ACT_LEAKY else (0.0 if act == ACT_RELU else 1.0)
    t = dz.interior + (dz2.interior if dz2 is not None else 0.0)
    g = dz.like(dz.a.shape[1], g_halo[0], g_halo[1], fill=0.0)
    g.interior[...] = t * np.where(z.interior > 0, 1.0, slope)
    return g


def pool3d_fwd(x: Slab, mode: int, y_halo=(0, 0)) -> Slab:
    """2x2x2 stride-2 pooling of the interior (Table I: stride-2 pooling)."""
    n, c, _, h, w = x.a.shape
    y = Slab(np.zeros((n, c, y_halo[0] + x.d // 2 + y_halo[1], h // 2, w // 2)), y_halo[0], y_halo[1],
             x.d_offset // 2, x.d_global // 2)
    _chk(_L().orc_pool3d_fwd(_p(x.a), x.geom(), _p(y.a), y.geom(), int(mode)), "pool3d_fwd")
    return y


def pool3d_bwd(dy: Slab, x: Slab | None, mode: int, dx_halo=(0, 0)) -> Slab:
    n, c, _, h, w = dy.a.shape
    dx = Slab(np.zeros((n, c, dx_halo[0] + 2 * dy.d + dx_halo[1], 2 * h, 2 * w)), dx_halo[0], dx_halo[1],
              dy.d_offset * 2, dy.d_global * 2)
    _chk(_L().orc_pool3d_bwd(_p(dy.a), dy.geom(), _p(x.a) if x is not None else None,
                             x.geom() if x is not None else None, _p(dx.a), dx.geom(), int(mode)), "pool3d_bwd")
    return dx


def deconv2_fwd(x: Slab, w, bias) -> Slab:
    """2x2x2 stride-2 transposed convolution, w [cin][cout][2][2][2] (U-Net up-sampling, Sec. II-C)."""
    w = _f64(w)
    bias = _f64(bias)
    n, c, _, h, ww = x.a.shape
    assert w.shape == (c, w.shape[1], 2, 2, 2)
    y = Slab(np.zeros((n, w.shape[1], 2 * x.d, 2 * h, 2 * ww)), 0, 0, 2 * x.d_offset, 2 * x.d_global)
    xi = Slab(x.interior, 0, 0, x.d_offset, x.d_global)
    _chk(_L().orc_deconv2_fwd(_p(xi.a), xi.geom(), _p(w), _p(bias), _p(y.a), y.geom()), "deconv2_fwd")
    return y


def deconv2_bwd_data(dy: Slab, w) -> Slab:
    w = _f64(w)
    n, c, _, h, ww = dy.a.shape
    dyi = Slab(dy.interior, 0, 0, dy.d_offset, dy.d_global)
    dx = Slab(np.zeros((n, w.shape[0], dy.d // 2, h // 2, ww // 2)), 0, 0, dy.d_offset // 2, dy.d_global // 2)
    _chk(_L().orc_deconv2_bwd_data(_p(dyi.a), dyi.geom(), _p(w), _p(dx.a), dx.geom()), "deconv2_bwd_data")
    return dx


def deconv2_bwd_filter(x: Slab, dy: Slab):
    xi = Slab(x.interior, 0, 0, x.d_offset, x.d_global)
    dyi = Slab(dy.interior, 0, 0, dy.d_offset, dy.d_global)
    cin, cout = xi.a.shape[1], dyi.a.shape[1]
    dw = np.zeros((cin, cout, 2, 2, 2))
    db = np.zeros((cout,))
    _chk(_L().orc_deconv2_bwd_filter(_p(xi.a), xi.geom(), _p(dyi.a), dyi.geom(), _p(dw), _p(db)), "deconv2_bwd_filter")
    return dw, db


# ------------------------------------------------------------ index-only steps (numpy slicing)

def halo_pack(t: Slab, face: int, width: int) -> np.ndarray:
    """The `width` outermost INTERIOR planes next to `face`, as [n][c][width][h][w] (Sec. III-A pack kernels)."""
    assert 0 < width <= t.d
    lo = t.halo_lo if face == FACE_D_LO else t.halo_lo + t.d - width
    return t.a[:, :, lo:lo + width].copy()


def halo_unpack(buf: np.ndarray | None, t: Slab, face: int, width: int) -> None:
    """Write `buf` (or zeros: global boundary) into the `width` HALO planes adjacent to the interior at `face`."""
    if face == FACE_D_LO:
        assert width <= t.halo_lo
        lo = t.halo_lo - width
    else:
        assert width <= t.halo_hi
        lo = t.halo_lo + t.d
    t.a[:, :, lo:lo + width] = 0.0 if buf is None else buf


def act_mask(z: Slab) -> np.ndarray:
    """Sign mask of a saved activation output (the derivative of ReLU / leaky ReLU only needs z > 0, Sec. IV-A's
    activations): uint8 [n][c][d][h][w/8] over the interior planes, bit k of byte j of a row = (z[8 j + k] > 0)."""
    zi = z.interior
    assert zi.shape[4] % 8 == 0
    out = np.zeros(zi.shape[:4] + (zi.shape[4] // 8,), dtype=np.uint8)
    for k in range(8):
        out |= (zi[..., k::8] > 0).astype(np.uint8) << k
    return out


def box_pack(a: np.ndarray, box) -> np.ndarray:
    """General face (Sec. II-B partitioning in any spatial dimension, Sec. III-A pack kernels): the box
    (d0, h0, w0, bd, bh, bw) of every (n, c) volume of the packed array a[n][c][D][H][W], as [n][c][bd][bh][bw]."""
    d0, h0, w0, bd, bh, bw = box
    assert a.ndim == 5 and 0 <= d0 and d0 + bd <= a.shape[2] and 0 <= h0 and h0 + bh <= a.shape[3] and 0 <= w0 and w0 + bw <= a.shape[4]
    out = np.empty((a.shape[0], a.shape[1], bd, bh, bw), dtype=a.dtype)
    for d in range(bd):
        for h in range(bh):
            for w in range(bw):
                out[:, :, d, h, w] = a[:, :, d0 + d, h0 + h, w0 + w]
    return out


def box_unpack(buf: np.ndarray | None, a: np.ndarray, box) -> None:
    """Write buf[n][c][bd][bh][bw] (or zeros: a face on the global boundary) into the box of a; the rest of a stays."""
    d0, h0, w0, bd, bh, bw = box
    assert a.ndim == 5 and 0 <= d0 and d0 + bd <= a.shape[2] and 0 <= h0 and h0 + bh <= a.shape[3] and 0 <= w0 and w0 + bw <= a.shape[4]
    for d in range(bd):
        for h in range(bh):
            for w in range(bw):
                a[:, :, d0 + d, h0 + h, w0 + w] = 0.0 if buf is None else buf[:, :, d, h, w]


def concat_c(a: Slab, b: Slab) -> Slab:
    """Channel concat of the interiors, `a` first (skip connection of the U-Net, Sec. III-A)."""
    return Slab(np.concatenate([a.interior, b.interior], axis=1), 0, 0, a.d_offset, a.d_global)


def split_c(g: Slab, ca: int):
    gi = g.interior
    return (Slab(gi[:, :ca].copy(), 0, 0, g.d_offset, g.d_global), Slab(gi[:, ca:].copy(), 0, 0, g.d_offset, g.d_global))


# ------------------------------------------------------------ dense / loss (library matmul as the step)

def _act(y, act, alpha):
    if act == ACT_NONE:
        return y
    s = alpha if act == ACT_LEAKY else 0.0
    return np.where(y > 0, y, s * y)


def dense_fwd(x, w, b, act=ACT_NONE, alpha=0.0):
    """y = act(x W^T + b); x [m,k], W [n,k] (fully-connected layers of Table I)."""
    y = _f64(x) @ _f64(w).T
    if b is not None:
        y = y + _f64(b)
    return _act(y, act, alpha)


def dense_bwd(x, w, y, dy, act=ACT_NONE, alpha=0.0):
    """Returns dx [m,k], dW [n,k], db [n]; `y` is the saved activated output."""
    g = _f64(dy)
    if act != ACT_NONE:
        s = alpha if act == ACT_LEAKY else 0.0
        g = g * np.where(_f64(y) > 0, 1.0, s)
    return g @ _f64(w), g.T @ _f64(x), g.sum(axis=0)


def mse_fwd_bwd(pred, target):
    """Mean squared error over all entries (Sec. IV: loss) and its gradient."""
    p, t = _f64(pred), _f64(target)
    diff = p - t
    return float(np.mean(diff * diff)), 2.0 * diff / diff.size


# ------------------------------------------------------------ batch normalisation, the local parts (Sec. II-B, III-C)
# Distributed batch normalisation = per-shard partial sums, an allreduce over the shards (not part of this
# code), then a per-channel affine map.  "Local" means: sums over the interior planes of THIS slab only.

def bn_stats(x: Slab):
    """Per-channel partial statistics of the slab's interior: (sum x, sum x^2), each [C]."""
    a = _f64(x.interior)
    return a.sum(axis=(0, 2, 3, 4)), (a * a).sum(axis=(0, 2, 3, 4))


def bn_finalize(s, sq, count: int, eps: float):
    """Mean and 1/sqrt(var + eps) (biased variance, as in training) from the summed statistics of `count` voxels."""
    mean = _f64(s) / count
    var = _f64(sq) / count - mean * mean
    return mean, 1.0 / np.sqrt(var + eps)


def bn_fwd(x: Slab, mean, invstd, gamma, beta) -> Slab:
    """y = gamma * (x - mean) * invstd + beta on the interior; halo planes of y are left zero."""
    y = x.like(x.a.shape[1], 0, 0)
    sh = (1, -1, 1, 1, 1)
    y.a[...] = _f64(gamma).reshape(sh) * (_f64(x.interior) - _f64(mean).reshape(sh)) * _f64(invstd).reshape(sh) + _f64(beta).reshape(sh)
    return y


def bn_bwd_stats(dy: Slab, x: Slab, mean, invstd):
    """Per-channel partial sums of the backward pass: (sum dy, sum dy * xhat) = (dbeta, dgamma) partials."""
    sh = (1, -1, 1, 1, 1)
    g = _f64(dy.interior)
    xhat = (_f64(x.interior) - _f64(mean).reshape(sh)) * _f64(invstd).reshape(sh)
    return g.sum(axis=(0, 2, 3, 4)), (g * xhat).sum(axis=(0, 2, 3, 4))


def bn_bwd(dy: Slab, x: Slab, mean, invstd, gamma, sum_dy, sum_dy_xhat, count: int) -> Slab:
    """dx = gamma * invstd * (dy - sum_dy / count - xhat * sum_dy_xhat / count), sums taken over all shards."""
    sh = (1, -1, 1, 1, 1)
    xhat = (_f64(x.interior) - _f64(mean).reshape(sh)) * _f64(invstd).reshape(sh)
    dx = x.like(x.a.shape[1], 0, 0)
    dx.a[...] = (_f64(gamma) * _f64(invstd)).reshape(sh) * (
        _f64(dy.interior) - (_f64(sum_dy) / count).reshape(sh) - xhat * (_f64(sum_dy_xhat) / count).reshape(sh))
    return dx


def num_threads() -> int:
    return int(_L().orc_num_threads())


# ------------------------------------------------------------ bookkeeping pinned by Table I

def conv_flops(cin: int, cout: int, out_voxels: int, k: int = 3) -> int:
    """2 * k^3 * Cin * Cout per output voxel (convention fixed by Table I's conv-op counts)."""
    return 2 * k ** 3 * cin * cout * out_voxels
