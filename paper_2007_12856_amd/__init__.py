"""Python binding of libh3d (the C ABI declared in include/h3d.h).

Argument marshalling only: every function here builds the C descriptors and
calls the entry point of the same name; all arithmetic runs in the HIP kernels.
PyTorch is used for device memory (`tensor.data_ptr()`) and the current stream.
There is no CPU or PyTorch fallback: if libh3d.so is missing or a call fails,
an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libh3d.so")

F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_LEAKY = 0, 1, 2
POOL_AVG, POOL_MAX = 0, 1
FACE_D_LO, FACE_D_HI, FACE_D_BOTH = 0, 1, 2
OP_FWD, OP_BWD_DATA, OP_BWD_FILTER = 0, 1, 2
STATUS = {0: "H3D_OK", -1: "H3D_EINVAL", -2: "H3D_EUNSUPPORTED", -3: "H3D_EWORKSPACE", -4: "H3D_EHALO", -5: "H3D_EHIP"}


class H3DError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class h3d_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("n", ctypes.c_int32), ("c", ctypes.c_int32),
                ("d", ctypes.c_int32), ("h", ctypes.c_int32), ("w", ctypes.c_int32), ("halo_lo", ctypes.c_int32),
                ("halo_hi", ctypes.c_int32), ("d_offset", ctypes.c_int64), ("d_global", ctypes.c_int64),
                ("c_stride", ctypes.c_int64), ("n_stride", ctypes.c_int64)]


class h3d_box(ctypes.Structure):
    _fields_ = [("d0", ctypes.c_int32), ("h0", ctypes.c_int32), ("w0", ctypes.c_int32),
                ("bd", ctypes.c_int32), ("bh", ctypes.c_int32), ("bw", ctypes.c_int32)]


_lib = None
_P = ctypes.c_void_p
_T = ctypes.POINTER(h3d_tensor)
_B = ctypes.POINTER(h3d_box)
_SIGNATURES = {
    "h3d_create": (ctypes.c_int, [ctypes.POINTER(_P)]),
    "h3d_destroy": (ctypes.c_int, [_P]),
    "h3d_last_error": (ctypes.c_char_p, [_P]),
    "h3d_last_kernel": (ctypes.c_char_p, [_P]),
    "h3d_conv3d_workspace_bytes": (ctypes.c_size_t, [_P, ctypes.c_int, _T, _T]),
    "h3d_conv3d_fwd": (ctypes.c_int, [_P, _T, _P, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_bwd_data": (ctypes.c_int, [_P, _T, _T, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_bwd_filter": (ctypes.c_int, [_P, _T, _T, _T, _P, _P, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_static_scratch_bytes": (ctypes.c_size_t, []),
    "h3d_conv3d_bwd_filter_static": (ctypes.c_int, [_P, _T, _T, _T, _P, _P, ctypes.c_int, ctypes.c_float, _P]),
    "h3d_conv3d_s2_workspace_bytes": (ctypes.c_size_t, [_P, ctypes.c_int, _T, _T]),
    "h3d_conv3d_s2_fwd": (ctypes.c_int, [_P, _T, _P, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_s2_bwd_data": (ctypes.c_int, [_P, _T, _T, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_s2_bwd_filter": (ctypes.c_int, [_P, _T, _T, _T, _P, _P, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_k5_workspace_bytes": (ctypes.c_size_t, [_P, ctypes.c_int, _T, _T]),
    "h3d_conv3d_k5_fwd": (ctypes.c_int, [_P, _T, _P, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_k5_bwd_data": (ctypes.c_int, [_P, _T, _T, _P, _T, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_conv3d_k5_bwd_filter": (ctypes.c_int, [_P, _T, _T, _T, _P, _P, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_act_bwd": (ctypes.c_int, [_P, _T, _T, _T, _T, ctypes.c_int, ctypes.c_float, _P]),
    "h3d_pool3d_fwd": (ctypes.c_int, [_P, _T, _T, ctypes.c_int, _P]),
    "h3d_pool3d_bwd": (ctypes.c_int, [_P, _T, _T, _T, ctypes.c_int, _P]),
    "h3d_pool3d_bwd_act": (ctypes.c_int, [_P, _T, _T, _T, _T, _T, ctypes.c_int, ctypes.c_int, ctypes.c_float, _P]),
    "h3d_pool3d_fwd_mask": (ctypes.c_int, [_P, _T, _T, _P, _P]),
    "h3d_act_mask_bytes": (ctypes.c_size_t, [_T]),
    "h3d_conv3d_fwd_pool": (ctypes.c_int, [_P, _T, _P, _P, _T, _T, _P, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t, _P]),
    "h3d_act_mask": (ctypes.c_int, [_P, _T, _P, _P]),
    "h3d_pool3d_bwd_mask": (ctypes.c_int, [_P, _T, _P, _T, ctypes.c_int, ctypes.c_float, _P]),
    "h3d_halo_bytes": (ctypes.c_size_t, [_T, ctypes.c_int]),
    "h3d_halo_pack": (ctypes.c_int, [_P, _T, ctypes.c_int, ctypes.c_int, _P, _P]),
    "h3d_halo_unpack": (ctypes.c_int, [_P, _P, _T, ctypes.c_int, ctypes.c_int, _P]),
    "h3d_box_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_int, ctypes.c_int, _B]),
    "h3d_box_pack": (ctypes.c_int, [_P, _P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    _B, _P, _P]),
    "h3d_box_unpack": (ctypes.c_int, [_P, _P, _P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, _B, _P]),
    "h3d_deconv2_workspace_bytes": (ctypes.c_size_t, [_P, ctypes.c_int, _T, _T]),
    "h3d_deconv2_fwd": (ctypes.c_int, [_P, _T, _P, _P, _T, _P, ctypes.c_size_t, _P]),
    "h3d_deconv2_bwd_data": (ctypes.c_int, [_P, _T, _P, _T, _P, ctypes.c_size_t, _P]),
    "h3d_deconv2_bwd_filter": (ctypes.c_int, [_P, _T, _T, _P, _P, _P, ctypes.c_size_t, _P]),
    "h3d_concat_c": (ctypes.c_int, [_P, _T, _T, _T, _P]),
    "h3d_split_c": (ctypes.c_int, [_P, _T, _T, _T, _P]),
    "h3d_dense_fwd": (ctypes.c_int, [_P, _P, _P, _P, _P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_float, _P]),
    "h3d_dense_bwd": (ctypes.c_int, [_P, _P, _P, _P, _P, _P, _P, _P, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_float, _P]),
    "h3d_mse_fwd_bwd": (ctypes.c_int, [_P, _P, _P, _P, _P, ctypes.c_int, ctypes.c_int, _P]),
    "h3d_bn_workspace_bytes": (ctypes.c_size_t, [_P, _T]),
    "h3d_bn_stats": (ctypes.c_int, [_P, _T, _P, _P, _P, ctypes.c_size_t, _P]),
    "h3d_bn_finalize": (ctypes.c_int, [_P, _P, _P, ctypes.c_int, ctypes.c_int64, ctypes.c_float, _P, _P, _P]),
    "h3d_bn_fwd": (ctypes.c_int, [_P, _T, _P, _P, _P, _P, _T, _P, ctypes.c_size_t, _P]),
    "h3d_bn_bwd_stats": (ctypes.c_int, [_P, _T, _T, _P, _P, _P, _P, _P, ctypes.c_size_t, _P]),
    "h3d_bn_bwd": (ctypes.c_int, [_P, _T, _T, _P, _P, _P, _P, _P, ctypes.c_int64, _T, _P, ctypes.c_size_t, _P]),
}


def lib():
    """The loaded C library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2007_12856_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


_handle = None


def h3d_create():
    """A new library handle (host object; bound to the current device)."""
    h = _P()
    st = lib().h3d_create(ctypes.byref(h))
    if st != 0:
        raise H3DError(st, "h3d_create failed")
    return h


def h3d_destroy(h) -> None:
    st = lib().h3d_destroy(h)
    if st != 0:
        raise H3DError(st, "h3d_destroy failed")


def h3d_last_error(h=None) -> str:
    return (lib().h3d_last_error(h if h is not None else handle()) or b"").decode()


def h3d_last_kernel(h=None) -> str:
    """Name of the kernel that did the arithmetic of the last compute call (for the benchmark's per-kernel table)."""
    return (lib().h3d_last_kernel(h if h is not None else handle()) or b"").decode()


def handle():
    """The module-wide handle the wrappers below use."""
    global _handle
    if _handle is None:
        _handle = h3d_create()
    return _handle


def _check(st: int):
    if st != 0:
        raise H3DError(st, h3d_last_error())


def _stream():
    import torch
    return _P(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else _P(t.data_ptr())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


@dataclass
class Slab:
    """A depth slab: `t` is a device tensor [N, C, halo_lo + d + halo_hi, H, W], either contiguous or a run of planes
    sliced out of a taller contiguous slab (`planes()`: the convolution passes accept such views)."""
    t: object
    halo_lo: int = 0
    halo_hi: int = 0
    d_offset: int = 0
    d_global: int | None = None

    def __post_init__(self):
        assert self.t.dim() == 5
        n, c, ds, h, w = self.t.shape
        assert self.t.is_contiguous() or self.t.stride()[2:] == (h * w, w, 1), "only whole planes can be sliced"
        if self.d_global is None:
            self.d_global = self.d

    @property
    def d(self) -> int:
        return self.t.shape[2] - self.halo_lo - self.halo_hi

    @property
    def interior(self):
        return self.t[:, :, self.halo_lo:self.halo_lo + self.d]

    def desc(self) -> h3d_tensor:
        n, c, _, h, w = self.t.shape
        cs, ns = (0, 0) if self.t.is_contiguous() else (self.t.stride(1), self.t.stride(0))
        return h3d_tensor(self.t.data_ptr(), _dtype_code(self.t), n, c, self.d, h, w, self.halo_lo, self.halo_hi,
                          self.d_offset, self.d_global, cs, ns)

    def planes(self, p0: int, p1: int, halo_lo: int = 0, halo_hi: int = 0) -> "Slab":
        """The interior planes [p0, p1) of this slab (indices relative to its first interior plane; they may reach
        into its halo) as a view with the given halo widths: no copy, same memory."""
        a, b = self.halo_lo + p0 - halo_lo, self.halo_lo + p1 + halo_hi
        assert 0 <= a <= b <= self.t.shape[2]
        return Slab(self.t[:, :, a:b], halo_lo, halo_hi, self.d_offset + p0, self.d_global)

    def channels(self, c0: int, c1: int, halo_lo: int | None = None, halo_hi: int | None = None) -> "Slab":
        """Channels [c0, c1) of this slab as a view (no copy, same memory), optionally with narrower halos: the planes
        dropped from the halo are simply not part of the view."""
        hl = self.halo_lo if halo_lo is None else halo_lo
        hh = self.halo_hi if halo_hi is None else halo_hi
        assert 0 <= c0 <= c1 <= self.t.shape[1] and hl <= self.halo_lo and hh <= self.halo_hi
        a, b = self.halo_lo - hl, self.t.shape[2] - (self.halo_hi - hh)
        return Slab(self.t[:, c0:c1, a:b], hl, hh, self.d_offset, self.d_global)

    def like(self, channels: int, halo_lo: int = 0, halo_hi: int = 0, d: int | None = None, h: int | None = None,
             w: int | None = None, d_offset: int | None = None, d_global: int | None = None) -> "Slab":
        import torch
        n, _, _, hh, ww = self.t.shape
        d = self.d if d is None else d
        t = torch.empty((n, channels, halo_lo + d + halo_hi, hh if h is None else h, ww if w is None else w),
                        dtype=self.t.dtype, device=self.t.device)
        return Slab(t, halo_lo, halo_hi, self.d_offset if d_offset is None else d_offset,
                    self.d_global if d_global is None else d_global)


class Workspace:
    """A caller-owned, growable device scratch buffer handed to the calls that need one."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes: int):
        import torch
        if nbytes <= 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
        return _P(self.buf.data_ptr()), int(self.buf.numel())


_ws = Workspace()


# ---------------------------------------------------------------- entry points (same names as the C ABI)

def h3d_conv3d_workspace_bytes(op: int, x: Slab, z: Slab) -> int:
    return int(lib().h3d_conv3d_workspace_bytes(handle(), op, ctypes.byref(x.desc()), ctypes.byref(z.desc())))


def h3d_conv3d_fwd(x: Slab, w, bias, z: Slab, act: int = ACT_NONE, alpha: float = 0.0, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_workspace_bytes(OP_FWD, x, z))
    _check(lib().h3d_conv3d_fwd(handle(), ctypes.byref(x.desc()), _ptr(w), _ptr(bias), ctypes.byref(z.desc()), act,
                                alpha, p, n, _stream()))
    return z


def _z_desc(x: Slab, z) -> h3d_tensor:
    """Descriptor of the unpooled output: a Slab, or its shape (n, c, d, h, w) alone when it is not to be stored."""
    if isinstance(z, Slab):
        return z.desc()
    n, c, d, h, w = (int(v) for v in z)
    return h3d_tensor(None, _dtype_code(x.t), n, c, d, h, w, 0, 0, x.d_offset, x.d_global, 0, 0)


def h3d_act_mask_bytes(x: Slab, z) -> int:
    return int(lib().h3d_act_mask_bytes(ctypes.byref(_z_desc(x, z))))


def h3d_conv3d_fwd_pool(x: Slab, w, bias, z, y: Slab, mask, act: int = ACT_NONE, alpha: float = 0.0, ws: Workspace | None = None):
    zd = _z_desc(x, z)
    nbytes = int(lib().h3d_conv3d_workspace_bytes(handle(), OP_FWD, ctypes.byref(x.desc()), ctypes.byref(zd)))
    p, n = (ws or _ws).get(nbytes)
    _check(lib().h3d_conv3d_fwd_pool(handle(), ctypes.byref(x.desc()), _ptr(w), _ptr(bias), ctypes.byref(zd), ctypes.byref(y.desc()),
                                     _ptr(mask), act, alpha, p, n, _stream()))
    return y


def h3d_act_mask(z: Slab, mask):
    _check(lib().h3d_act_mask(handle(), ctypes.byref(z.desc()), _ptr(mask), _stream()))
    return mask


def h3d_pool3d_fwd_mask(x: Slab, y: Slab, mask):
    _check(lib().h3d_pool3d_fwd_mask(handle(), ctypes.byref(x.desc()), ctypes.byref(y.desc()), _ptr(mask), _stream()))
    return y


def h3d_pool3d_bwd_mask(dy: Slab, mask, g: Slab, act: int, alpha: float = 0.0):
    _check(lib().h3d_pool3d_bwd_mask(handle(), ctypes.byref(dy.desc()), _ptr(mask), ctypes.byref(g.desc()), act, alpha, _stream()))
    return g


def h3d_conv3d_bwd_data(dz: Slab, z: Slab | None, w, dx: Slab, act: int = ACT_NONE, alpha: float = 0.0,
                        ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_workspace_bytes(OP_BWD_DATA, dz, dx))
    _check(lib().h3d_conv3d_bwd_data(handle(), ctypes.byref(dz.desc()), ctypes.byref(z.desc()) if z is not None else None,
                                     _ptr(w), ctypes.byref(dx.desc()), act, alpha, p, n, _stream()))
    return dx


def h3d_conv3d_bwd_filter(x: Slab, dz: Slab, z: Slab | None, dw, db, act: int = ACT_NONE, alpha: float = 0.0,
                          ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_workspace_bytes(OP_BWD_FILTER, x, dz))
    _check(lib().h3d_conv3d_bwd_filter(handle(), ctypes.byref(x.desc()), ctypes.byref(dz.desc()),
                                       ctypes.byref(z.desc()) if z is not None else None, _ptr(dw), _ptr(db), act, alpha,
                                       p, n, _stream()))
    return dw, db


def h3d_static_scratch_bytes() -> int:
    return int(lib().h3d_static_scratch_bytes())


def h3d_conv3d_bwd_filter_static(x: Slab, dz: Slab, z: Slab | None, dw, db, act: int = ACT_NONE, alpha: float = 0.0):
    """Backward-filter on the library's own scratch array: no workspace is passed, nothing is allocated."""
    _check(lib().h3d_conv3d_bwd_filter_static(handle(), ctypes.byref(x.desc()), ctypes.byref(dz.desc()),
                                              ctypes.byref(z.desc()) if z is not None else None, _ptr(dw), _ptr(db), act, alpha,
                                              _stream()))
    return dw, db


def h3d_conv3d_s2_workspace_bytes(op: int, x: Slab, y: Slab) -> int:
    return int(lib().h3d_conv3d_s2_workspace_bytes(handle(), op, ctypes.byref(x.desc()), ctypes.byref(y.desc())))


def h3d_conv3d_s2_fwd(x: Slab, w, bias, y: Slab, act: int = ACT_NONE, alpha: float = 0.0, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_s2_workspace_bytes(OP_FWD, x, y))
    _check(lib().h3d_conv3d_s2_fwd(handle(), ctypes.byref(x.desc()), _ptr(w), _ptr(bias), ctypes.byref(y.desc()), act,
                                   alpha, p, n, _stream()))
    return y


def h3d_conv3d_s2_bwd_data(dy: Slab, y: Slab | None, w, dx: Slab, act: int = ACT_NONE, alpha: float = 0.0,
                           ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_s2_workspace_bytes(OP_BWD_DATA, dx, dy))
    _check(lib().h3d_conv3d_s2_bwd_data(handle(), ctypes.byref(dy.desc()), ctypes.byref(y.desc()) if y is not None else None,
                                        _ptr(w), ctypes.byref(dx.desc()), act, alpha, p, n, _stream()))
    return dx


def h3d_conv3d_s2_bwd_filter(x: Slab, dy: Slab, y: Slab | None, dw, db, act: int = ACT_NONE, alpha: float = 0.0,
                             ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_s2_workspace_bytes(OP_BWD_FILTER, x, dy))
    _check(lib().h3d_conv3d_s2_bwd_filter(handle(), ctypes.byref(x.desc()), ctypes.byref(dy.desc()),
                                          ctypes.byref(y.desc()) if y is not None else None, _ptr(dw), _ptr(db), act, alpha,
                                          p, n, _stream()))
    return dw, db


def h3d_conv3d_k5_workspace_bytes(op: int, x: Slab, z: Slab) -> int:
    return int(lib().h3d_conv3d_k5_workspace_bytes(handle(), op, ctypes.byref(x.desc()), ctypes.byref(z.desc())))


def h3d_conv3d_k5_fwd(x: Slab, w, bias, z: Slab, act: int = ACT_NONE, alpha: float = 0.0, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_k5_workspace_bytes(OP_FWD, x, z))
    _check(lib().h3d_conv3d_k5_fwd(handle(), ctypes.byref(x.desc()), _ptr(w), _ptr(bias), ctypes.byref(z.desc()), act,
                                   alpha, p, n, _stream()))
    return z


def h3d_conv3d_k5_bwd_data(dz: Slab, z: Slab | None, w, dx: Slab, act: int = ACT_NONE, alpha: float = 0.0,
                           ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_k5_workspace_bytes(OP_BWD_DATA, dx, dz))
    _check(lib().h3d_conv3d_k5_bwd_data(handle(), ctypes.byref(dz.desc()), ctypes.byref(z.desc()) if z is not None else None,
                                        _ptr(w), ctypes.byref(dx.desc()), act, alpha, p, n, _stream()))
    return dx


def h3d_conv3d_k5_bwd_filter(x: Slab, dz: Slab, z: Slab | None, dw, db, act: int = ACT_NONE, alpha: float = 0.0,
                             ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_conv3d_k5_workspace_bytes(OP_BWD_FILTER, x, dz))
    _check(lib().h3d_conv3d_k5_bwd_filter(handle(), ctypes.byref(x.desc()), ctypes.byref(dz.desc()),
                                          ctypes.byref(z.desc()) if z is not None else None, _ptr(dw), _ptr(db), act, alpha,
                                          p, n, _stream()))
    return dw, db


def h3d_act_bwd(dz: Slab, dz2: Slab | None, z: Slab, g: Slab, act: int, alpha: float = 0.0):
    _check(lib().h3d_act_bwd(handle(), ctypes.byref(dz.desc()), ctypes.byref(dz2.desc()) if dz2 is not None else None,
                             ctypes.byref(z.desc()), ctypes.byref(g.desc()), act, alpha, _stream()))
    return g


def h3d_pool3d_fwd(x: Slab, y: Slab, mode: int):
    _check(lib().h3d_pool3d_fwd(handle(), ctypes.byref(x.desc()), ctypes.byref(y.desc()), mode, _stream()))
    return y


def h3d_pool3d_bwd(dy: Slab, x: Slab | None, dx: Slab, mode: int):
    _check(lib().h3d_pool3d_bwd(handle(), ctypes.byref(dy.desc()), ctypes.byref(x.desc()) if x is not None else None,
                                ctypes.byref(dx.desc()), mode, _stream()))
    return dx


def h3d_pool3d_bwd_act(dy: Slab, x: Slab | None, z: Slab, g: Slab, mode: int, act: int, alpha: float = 0.0, dz2: Slab | None = None):
    _check(lib().h3d_pool3d_bwd_act(handle(), ctypes.byref(dy.desc()), ctypes.byref(x.desc()) if x is not None else None,
                                    ctypes.byref(z.desc()), ctypes.byref(dz2.desc()) if dz2 is not None else None,
                                    ctypes.byref(g.desc()), mode, act, alpha, _stream()))
    return g


def h3d_halo_bytes(t: Slab, width: int) -> int:
    return int(lib().h3d_halo_bytes(ctypes.byref(t.desc()), width))


def h3d_halo_pack(t: Slab, face: int, width: int, buf):
    _check(lib().h3d_halo_pack(handle(), ctypes.byref(t.desc()), face, width, _ptr(buf), _stream()))
    return buf


def h3d_halo_unpack(buf, t: Slab, face: int, width: int):
    _check(lib().h3d_halo_unpack(handle(), _ptr(buf), ctypes.byref(t.desc()), face, width, _stream()))
    return t


def _box_args(t, box):
    """t: contiguous 5-D torch tensor [n][c][D][H][W] (stored extents); box = (d0, h0, w0, bd, bh, bw)."""
    import torch
    if t.dim() != 5 or not t.is_contiguous():
        raise ValueError("box_pack/unpack: a contiguous 5-D tensor is required")
    dt = {torch.float32: F32, torch.bfloat16: BF16}[t.dtype]
    n, c, D, H, W = (int(v) for v in t.shape)
    return dt, n, c, D, H, W, h3d_box(*[int(v) for v in box])


def h3d_box_bytes(t, box) -> int:
    dt, n, c, D, H, W, b = _box_args(t, box)
    return int(lib().h3d_box_bytes(dt, n, c, ctypes.byref(b)))


def h3d_box_pack(t, box, buf):
    dt, n, c, D, H, W, b = _box_args(t, box)
    _check(lib().h3d_box_pack(handle(), _ptr(t), dt, n, c, D, H, W, ctypes.byref(b), _ptr(buf), _stream()))
    return buf


def h3d_box_unpack(buf, t, box):
    dt, n, c, D, H, W, b = _box_args(t, box)
    _check(lib().h3d_box_unpack(handle(), _ptr(buf), _ptr(t), dt, n, c, D, H, W, ctypes.byref(b), _stream()))
    return t


def h3d_deconv2_workspace_bytes(op: int, x: Slab, y: Slab) -> int:
    return int(lib().h3d_deconv2_workspace_bytes(handle(), op, ctypes.byref(x.desc()), ctypes.byref(y.desc())))


def h3d_deconv2_fwd(x: Slab, w, bias, y: Slab, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_deconv2_workspace_bytes(OP_FWD, x, y))
    _check(lib().h3d_deconv2_fwd(handle(), ctypes.byref(x.desc()), _ptr(w), _ptr(bias), ctypes.byref(y.desc()), p, n, _stream()))
    return y


def h3d_deconv2_bwd_data(dy: Slab, w, dx: Slab, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_deconv2_workspace_bytes(OP_BWD_DATA, dx, dy))
    _check(lib().h3d_deconv2_bwd_data(handle(), ctypes.byref(dy.desc()), _ptr(w), ctypes.byref(dx.desc()), p, n, _stream()))
    return dx


def h3d_deconv2_bwd_filter(x: Slab, dy: Slab, dw, db, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_deconv2_workspace_bytes(OP_BWD_FILTER, x, dy))
    _check(lib().h3d_deconv2_bwd_filter(handle(), ctypes.byref(x.desc()), ctypes.byref(dy.desc()), _ptr(dw), _ptr(db), p, n, _stream()))
    return dw, db


def h3d_concat_c(a: Slab, b: Slab, out: Slab):
    _check(lib().h3d_concat_c(handle(), ctypes.byref(a.desc()), ctypes.byref(b.desc()), ctypes.byref(out.desc()), _stream()))
    return out


def h3d_split_c(inp: Slab, a: Slab, b: Slab):
    _check(lib().h3d_split_c(handle(), ctypes.byref(inp.desc()), ctypes.byref(a.desc()), ctypes.byref(b.desc()), _stream()))
    return a, b


def h3d_dense_fwd(x, w, bias, y, act: int = ACT_NONE, alpha: float = 0.0):
    m, k = x.shape
    n = w.shape[0]
    assert w.shape[1] == k and tuple(y.shape) == (m, n)
    _check(lib().h3d_dense_fwd(handle(), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _dtype_code(x), m, n, k, act, alpha, _stream()))
    return y


def h3d_dense_bwd(x, w, y, dy, dx, dw, db, act: int = ACT_NONE, alpha: float = 0.0):
    m, k = x.shape
    n = w.shape[0]
    _check(lib().h3d_dense_bwd(handle(), _ptr(x), _ptr(w), _ptr(y), _ptr(dy), _ptr(dx), _ptr(dw), _ptr(db), _dtype_code(x),
                               m, n, k, act, alpha, _stream()))
    return dx, dw, db


def h3d_mse_fwd_bwd(pred, target, loss, dpred):
    _check(lib().h3d_mse_fwd_bwd(handle(), _ptr(pred), _ptr(target), _ptr(loss), _ptr(dpred), _dtype_code(pred),
                                 pred.numel(), _stream()))
    return loss, dpred


def h3d_bn_workspace_bytes(x: Slab) -> int:
    return int(lib().h3d_bn_workspace_bytes(handle(), ctypes.byref(x.desc())))


def h3d_bn_stats(x: Slab, s, sq, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_bn_workspace_bytes(x))
    _check(lib().h3d_bn_stats(handle(), ctypes.byref(x.desc()), _ptr(s), _ptr(sq), p, n, _stream()))
    return s, sq


def h3d_bn_finalize(s, sq, count: int, eps: float, mean, invstd):
    _check(lib().h3d_bn_finalize(handle(), _ptr(s), _ptr(sq), s.numel(), int(count), float(eps), _ptr(mean), _ptr(invstd), _stream()))
    return mean, invstd


def h3d_bn_fwd(x: Slab, mean, invstd, gamma, beta, y: Slab, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_bn_workspace_bytes(x))
    _check(lib().h3d_bn_fwd(handle(), ctypes.byref(x.desc()), _ptr(mean), _ptr(invstd), _ptr(gamma), _ptr(beta),
                            ctypes.byref(y.desc()), p, n, _stream()))
    return y


def h3d_bn_bwd_stats(dy: Slab, x: Slab, mean, invstd, sum_dy, sum_dy_xhat, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_bn_workspace_bytes(x))
    _check(lib().h3d_bn_bwd_stats(handle(), ctypes.byref(dy.desc()), ctypes.byref(x.desc()), _ptr(mean), _ptr(invstd),
                                  _ptr(sum_dy), _ptr(sum_dy_xhat), p, n, _stream()))
    return sum_dy, sum_dy_xhat


def h3d_bn_bwd(dy: Slab, x: Slab, mean, invstd, gamma, sum_dy, sum_dy_xhat, count: int, dx: Slab, ws: Workspace | None = None):
    p, n = (ws or _ws).get(h3d_bn_workspace_bytes(x))
    _check(lib().h3d_bn_bwd(handle(), ctypes.byref(dy.desc()), ctypes.byref(x.desc()), _ptr(mean), _ptr(invstd), _ptr(gamma),
                            _ptr(sum_dy), _ptr(sum_dy_xhat), int(count), ctypes.byref(dx.desc()), p, n, _stream()))
    return dx


# short aliases
bn_stats, bn_finalize, bn_fwd, bn_bwd_stats, bn_bwd = h3d_bn_stats, h3d_bn_finalize, h3d_bn_fwd, h3d_bn_bwd_stats, h3d_bn_bwd
conv3d_fwd, conv3d_bwd_data, conv3d_bwd_filter = h3d_conv3d_fwd, h3d_conv3d_bwd_data, h3d_conv3d_bwd_filter
conv3d_bwd_filter_static, static_scratch_bytes = h3d_conv3d_bwd_filter_static, h3d_static_scratch_bytes
conv3d_s2_fwd, conv3d_s2_bwd_data, conv3d_s2_bwd_filter = h3d_conv3d_s2_fwd, h3d_conv3d_s2_bwd_data, h3d_conv3d_s2_bwd_filter
conv3d_k5_fwd, conv3d_k5_bwd_data, conv3d_k5_bwd_filter = h3d_conv3d_k5_fwd, h3d_conv3d_k5_bwd_data, h3d_conv3d_k5_bwd_filter
pool3d_fwd, pool3d_bwd, act_bwd, pool3d_bwd_act = h3d_pool3d_fwd, h3d_pool3d_bwd, h3d_act_bwd, h3d_pool3d_bwd_act
halo_bytes, halo_pack, halo_unpack = h3d_halo_bytes, h3d_halo_pack, h3d_halo_unpack
box_bytes, box_pack, box_unpack = h3d_box_bytes, h3d_box_pack, h3d_box_unpack
conv3d_fwd_pool, act_mask, act_mask_bytes, pool3d_bwd_mask = h3d_conv3d_fwd_pool, h3d_act_mask, h3d_act_mask_bytes, h3d_pool3d_bwd_mask
pool3d_fwd_mask = h3d_pool3d_fwd_mask
deconv2_fwd, deconv2_bwd_data, deconv2_bwd_filter = h3d_deconv2_fwd, h3d_deconv2_bwd_data, h3d_deconv2_bwd_filter
concat_c, split_c = h3d_concat_c, h3d_split_c
dense_fwd, dense_bwd, mse_fwd_bwd = h3d_dense_fwd, h3d_dense_bwd, h3d_mse_fwd_bwd
