"""Pins of the batch-normalisation oracle (local parts of distributed batch normalisation, Sec. II-B / III-C):
closed forms, invariants of the normalised output, shard additivity of the statistics (what makes the allreduce
correct), and a finite-difference check of the whole backward pass against the forward pass."""
import numpy as np

import oracle as orc
import synth

SEED = synth.BASE_SEED


def _slab(shape, stream, halo=(0, 0), off=0, dg=None):
    return orc.Slab(synth.flat("normal", SEED, stream, shape), halo[0], halo[1], off, dg)


def test_stats_closed_forms():
    # constant channel c holds the value c+1: sum = count*(c+1), sum of squares = count*(c+1)^2; halo planes are ignored
    a = np.empty((2, 3, 6, 4, 5))
    for c in range(3):
        a[:, c] = c + 1
    a[:, :, 0] = 99.0      # halo planes
    a[:, :, -1] = -99.0
    s, sq = orc.bn_stats(orc.Slab(a, 1, 1, 1, 6))
    count = 2 * 4 * 4 * 5
    assert np.allclose(s, count * np.array([1.0, 2.0, 3.0]))
    assert np.allclose(sq, count * np.array([1.0, 4.0, 9.0]))
    mean, invstd = orc.bn_finalize(s, sq, count, 1e-5)
    assert np.allclose(mean, [1, 2, 3]) and np.allclose(invstd, 1 / np.sqrt(1e-5))


def test_normalised_output_has_zero_mean_unit_variance_and_affine_is_applied():
    x = _slab((3, 4, 5, 6, 7), 1)
    count = 3 * 5 * 6 * 7
    s, sq = orc.bn_stats(x)
    mean, invstd = orc.bn_finalize(s, sq, count, 0.0)
    y = orc.bn_fwd(x, mean, invstd, np.ones(4), np.zeros(4))
    assert np.allclose(y.a.mean(axis=(0, 2, 3, 4)), 0, atol=1e-12)
    assert np.allclose(y.a.var(axis=(0, 2, 3, 4)), 1, atol=1e-10)
    gamma, beta = np.array([2.0, -1.0, 0.5, 3.0]), np.array([0.1, 0.2, -0.3, 4.0])
    y2 = orc.bn_fwd(x, mean, invstd, gamma, beta)
    assert np.allclose(y2.a, gamma.reshape(1, -1, 1, 1, 1) * y.a + beta.reshape(1, -1, 1, 1, 1))
    # against numpy's own moments (a library routine the oracle does not call)
    assert np.allclose(mean, x.a.mean(axis=(0, 2, 3, 4))) and np.allclose(1 / invstd ** 2, x.a.var(axis=(0, 2, 3, 4)))


def test_shard_statistics_add_up_to_the_whole():
    full = synth.flat("normal", SEED, 2, (2, 3, 8, 4, 5))
    whole = orc.bn_stats(orc.Slab(full))
    parts = [orc.bn_stats(orc.Slab(full[:, :, max(0, lo - 1):hi + 1], min(1, lo), 1 if hi < 8 else 0, lo, 8))
             for lo, hi in ((0, 3), (3, 5), (5, 8))]
    assert np.allclose(sum(p[0] for p in parts), whole[0]) and np.allclose(sum(p[1] for p in parts), whole[1])


def _bn_loss(xa, gamma, beta, r, eps):
    x = orc.Slab(xa)
    count = xa.size // xa.shape[1]
    mean, invstd = orc.bn_finalize(*orc.bn_stats(x), count, eps)
    return float((orc.bn_fwd(x, mean, invstd, gamma, beta).a * r).sum())


def test_backward_matches_finite_differences_of_the_forward():
    shape, eps = (2, 3, 3, 4, 5), 1e-3
    xa = synth.flat("normal", SEED, 3, shape)
    r = synth.flat("normal", SEED, 4, shape)           # dL/dy for L = sum(y * r)
    gamma, beta = np.array([1.5, -0.7, 0.9]), np.array([0.2, 0.0, -1.0])
    x, dy = orc.Slab(xa), orc.Slab(r)
    count = xa.size // 3
    mean, invstd = orc.bn_finalize(*orc.bn_stats(x), count, eps)
    sdy, sdyx = orc.bn_bwd_stats(dy, x, mean, invstd)
    dx = orc.bn_bwd(dy, x, mean, invstd, gamma, sdy, sdyx, count).a
    h = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(12):
        idx = tuple(rng.integers(0, s) for s in shape)
        xp, xm = xa.copy(), xa.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (_bn_loss(xp, gamma, beta, r, eps) - _bn_loss(xm, gamma, beta, r, eps)) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-6 * max(1.0, abs(fd))
    # dgamma = sum dy*xhat and dbeta = sum dy, by the same finite differences
    for c in range(3):
        gp, gm = gamma.copy(), gamma.copy()
        gp[c] += h
        gm[c] -= h
        assert abs((_bn_loss(xa, gp, beta, r, eps) - _bn_loss(xa, gm, beta, r, eps)) / (2 * h) - sdyx[c]) <= 1e-6 * max(1.0, abs(sdyx[c]))
        bp, bm = beta.copy(), beta.copy()
        bp[c] += h
        bm[c] -= h
        assert abs((_bn_loss(xa, gamma, bp, r, eps) - _bn_loss(xa, gamma, bm, r, eps)) / (2 * h) - sdy[c]) <= 1e-6 * max(1.0, abs(sdy[c]))
    # the gradient with respect to a normalised tensor sums to zero per channel
    assert np.allclose(dx.sum(axis=(0, 2, 3, 4)), 0, atol=1e-10)
