"""Seeded parameter / input recipes for the benchmark workloads (shapes and value ranges only).

Weights are uniform in +-sqrt(3/fan_in) so activations stay O(1) through a stack; conv biases
uniform in +-0.1; regression targets uniform in [-1,1] (the paper normalises the cosmological
parameters to that range, Sec. II-C).
"""
from __future__ import annotations

import numpy as np

from . import BASE_SEED, flat, slab

COSMO_CHANNELS = (4, 16, 32, 64, 128, 256)
COSMO_FC = (2048, 256, 4)


def conv_params(seed, stream, cin, cout, taps=27, transposed=False):
    b = float(np.sqrt(3.0 / (taps * cin)))
    k = (2, 2, 2) if taps == 8 else (3, 3, 3)
    shape = (cin, cout, *k) if transposed else (cout, cin, *k)
    w = flat("uniform", seed, stream, shape, -b, b)
    bias = flat("uniform", seed, stream + 1, (cout,), -0.1, 0.1)
    return w, bias


TABLE1_CHANNELS = (4, 16, 32, 64, 128, 256, 256, 256)
TABLE1_STRIDES = (1, 1, 1, 2, 1, 1, 1)


def table1_layout(width=128):
    """Channels, strides and pooling flags of the seven convolutions of Table I for a width^3 input
    (128, 256 or 512): every convolution is followed by a pooling until the volume is 2^3."""
    pools, w = [], width
    for st in TABLE1_STRIDES:
        w //= st
        pools.append(w > 2)
        if w > 2:
            w //= 2
    return TABLE1_CHANNELS, TABLE1_STRIDES, tuple(pools), TABLE1_CHANNELS[-1] * w ** 3


def cosmoflow_params(seed=BASE_SEED, width=128, channels=COSMO_CHANNELS, fc=COSMO_FC, flat_w=None):
    """{'conv': [(w,b)...], 'fc': [(w,b)...]} for the CosmoFlow-shaped stack on a width^3 input.
    flat_w: length of the flattened last activation (default: every stage halves the width once)."""
    conv = [conv_params(seed, 100 + 2 * i, channels[i], channels[i + 1]) for i in range(len(channels) - 1)]
    if flat_w is None:
        flat_w = channels[-1] * (width >> (len(channels) - 1)) ** 3
    dims = (flat_w, *fc)
    fcs = []
    for i in range(len(fc)):
        b = float(np.sqrt(3.0 / dims[i]))
        fcs.append((flat("uniform", seed, 200 + 2 * i, (dims[i + 1], dims[i]), -b, b),
                    flat("uniform", seed, 201 + 2 * i, (dims[i + 1],), -0.1, 0.1)))
    return {"conv": conv, "fc": fcs}


def cosmoflow_batch(seed=BASE_SEED, n=4, width=128, cin=4, nout=4):
    x = slab("cosmo", seed, 1, (n, cin, width, width, width), 0, width)
    t = flat("uniform", seed, 2, (n, nout), -1.0, 1.0)
    return x, t


UNET_WIDTHS = {"c1": (1, 32), "c2": (32, 64), "c3": (64, 64), "c4": (64, 128), "up": (128, 64), "c6": (128, 64)}


def unet_level_inputs(seed=BASE_SEED, d_global=256, d=64, d_offset=64, hw=256):
    """Inputs of one U-Net-shaped encoder/decoder level on a depth shard: the input slab with a
    2-plane halo cut from the seeded volume, the six layers' parameters, the upstream gradient, and
    the stand-in faces that a halo exchange with the two depth neighbours would deliver for the
    tensors whose halo cannot be recomputed locally (None at a global boundary)."""
    x = slab("normal", seed, 300, (1, 1, d_global, hw, hw), d_offset - 2, d_offset + d + 2)
    params = {}
    for i, (name, (ci, co)) in enumerate(UNET_WIDTHS.items()):
        params[name] = conv_params(seed, 310 + 2 * i, ci, co, taps=8 if name == "up" else 27, transposed=(name == "up"))
    dout = slab("normal", seed, 330, (1, 64, d_global, hw, hw), d_offset, d_offset + d)
    has_lo, has_hi = d_offset > 0, d_offset + d < d_global
    faces = {}
    spec = {"p": (64, 2, 2, True), "cat": (128, 1, 1, True), "g6": (64, 1, 1, False), "g4": (128, 1, 2, False),
            "g3": (64, 1, 2, False), "g2": (64, 1, 1, False), "g1": (32, 1, 1, False)}
    for k, (name, (c, width, level, nonneg)) in enumerate(spec.items()):
        s = hw // level
        lo = flat("normal", seed, 340 + 2 * k, (1, c, width, s, s)) if has_lo else None
        hi = flat("normal", seed, 341 + 2 * k, (1, c, width, s, s)) if has_hi else None
        if nonneg:   # these stand in for post-ReLU activations
            lo = None if lo is None else np.maximum(lo, 0.0)
            hi = None if hi is None else np.maximum(hi, 0.0)
        faces[name] = (lo, hi)
    return x, params, dout, faces


def shard_chain_inputs(seed=BASE_SEED, d_global=512, d=64, d_offset=64, hw=512, channels=(4, 16, 32, 64), n=1):
    """Inputs of the spatially-partitioned front of the Table I network on one depth shard: the input slab with a
    1-plane halo cut from the seeded volume, the stages' filters (no biases, Sec. IV), the gradient arriving at the
    last pooled tensor, and stand-in faces for what the two depth neighbours would send: 'a0' (the input's own halo
    planes), 'a1'.. (pooled activations), 'g1'.. (activation gradients); None at a global boundary."""
    x = slab("cosmo", seed, 400, (n, channels[0], d_global, hw, hw), d_offset - 1, d_offset + d + 1)
    conv = [(conv_params(seed, 410 + 2 * i, channels[i], channels[i + 1])[0], None) for i in range(len(channels) - 1)]
    L = len(conv)
    has_lo, has_hi = d_offset > 0, d_offset + d < d_global
    faces = {"a0": (x[:, :, :1].copy() if has_lo else None, x[:, :, -1:].copy() if has_hi else None)}
    for i in range(1, L + 1):
        s = hw >> (i - 1)
        for k, (name, c, width, scale) in enumerate((("a", channels[i], s // 2, 0.5), ("g", channels[i], s, 0.125))):
            if name == "a" and i == L:
                continue
            shape = (n, c, 1, width, width)
            lo = scale * flat("normal", seed, 420 + 8 * i + 4 * k, shape) if has_lo else None
            hi = scale * flat("normal", seed, 421 + 8 * i + 4 * k, shape) if has_hi else None
            faces[f"{name}{i}"] = (lo, hi)
    dl, sl = d >> L, hw >> L
    dout = slab("normal", seed, 490, (n, channels[-1], d_global >> L, sl, sl), d_offset >> L, (d_offset >> L) + dl)
    return x, conv, dout, faces
