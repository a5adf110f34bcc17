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


def cosmoflow_params(seed=BASE_SEED, width=128, channels=COSMO_CHANNELS, fc=COSMO_FC):
    """{'conv': [(w,b)...], 'fc': [(w,b)...]} for the CosmoFlow-shaped stack on a width^3 input."""
    conv = [conv_params(seed, 100 + 2 * i, channels[i], channels[i + 1]) for i in range(len(channels) - 1)]
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
