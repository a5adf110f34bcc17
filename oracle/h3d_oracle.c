/*
 * CPU oracle for the per-GPU layer computations of spatially-partitioned
 * 3-D CNN training (paper Sec. III-A: convolution and pooling on a depth
 * slab whose halo planes hold the neighbours' boundary data; Sec. III-C:
 * forward, backward-data and backward-filter passes per layer).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64, one direct loop nest per
 * definition; it shares no code with the HIP library and is never called by
 * the product path.  Only tests, the smoke check and the bench's CPU-baseline
 * leg may load it.
 *
 * Tensors are N,C,D,H,W, fully packed, W fastest (Sec. III "Notation").
 * A slab is described by nine int64: {n, c, d, h, w, halo_lo, halo_hi,
 * d_offset, d_global}.  Its buffer stores halo_lo + d + halo_hi depth planes;
 * interior plane p (0 <= p < d) is global plane d_offset + p of a sample whose
 * unsharded depth is d_global.  Everything outside the global volume
 * [0,d_global) x [0,h) x [0,w) is zero ("same" padding, Table I caption) and
 * is never read.
 *
 * The paper writes no convolution formula (it adopts the vendor library's
 * notation), so the definition here is the standard deep-learning
 * "convolution" = cross-correlation:
 *   y[n,co,p] = b[co] + sum_{ci,kd,kh,kw} w[co,ci,kd,kh,kw] * x~[n,ci,p+k-1]
 * with leaky-ReLU z = y > 0 ? y : alpha*y (Sec. IV, activations).
 *
 * Return value of every function: 0 ok, -1 bad argument, -4 a needed plane
 * inside the global volume is not stored in the slab.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { G_N = 0, G_C, G_D, G_H, G_W, G_HLO, G_HHI, G_DOFF, G_DGLOB };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_LEAKY = 2 };

static inline size_t at5(const int64_t* g, int64_t n, int64_t c, int64_t p, int64_t h, int64_t w) {
  /* p is the local interior plane index; stored plane = p + halo_lo */
  int64_t ds = g[G_HLO] + g[G_D] + g[G_HHI];
  return ((((size_t)n * g[G_C] + c) * ds + (p + g[G_HLO])) * g[G_H] + h) * g[G_W] + w;
}

static inline int stored(const int64_t* g, int64_t p) { return p >= -g[G_HLO] && p < g[G_D] + g[G_HHI]; }
static inline int in_volume(const int64_t* g, int64_t p) {
  int64_t q = g[G_DOFF] + p;
  return q >= 0 && q < g[G_DGLOB];
}

static inline double act_slope(int act, double alpha) {
  return act == ACT_LEAKY ? alpha : (act == ACT_RELU ? 0.0 : 1.0);
}

static int same_shard(const int64_t* a, const int64_t* b) {
  return a[G_N] == b[G_N] && a[G_D] == b[G_D] && a[G_H] == b[G_H] && a[G_W] == b[G_W] &&
         a[G_DOFF] == b[G_DOFF] && a[G_DGLOB] == b[G_DGLOB];
}

/* Which input planes does output range [lo,hi) need, and are they stored? */
static int halo_ok(const int64_t* in, int64_t lo, int64_t hi) {
  for (int64_t p = lo; p < hi; ++p) {
    if (!in_volume(in, p)) continue;
    for (int k = -1; k <= 1; ++k)
      if (in_volume(in, p + k) && !stored(in, p + k)) return 0;
  }
  return 1;
}

/* ------------------------------------------------------------------ forward */
/* z planes [-z.halo_lo, d + z.halo_hi) are produced; planes outside the global
 * volume are written as zero (they are the next layer's padding). */
int orc_conv3d_fwd(const double* x, const int64_t* xg, const double* w, const double* bias,
                   double* z, const int64_t* zg, int act, double alpha) {
  if (!same_shard(xg, zg)) return -1;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = zg[G_C], D = xg[G_D], H = xg[G_H], W = xg[G_W];
  const int64_t plo = -zg[G_HLO], phi = D + zg[G_HHI];
  if (!halo_ok(xg, plo, phi)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t co = 0; co < Co; ++co)
      for (int64_t p = plo; p < phi; ++p) {
        const int inside = in_volume(zg, p);
        for (int64_t h = 0; h < H; ++h)
          for (int64_t v = 0; v < W; ++v) {
            double acc = 0.0;
            if (inside) {
              acc = bias ? bias[co] : 0.0;
              for (int64_t ci = 0; ci < Ci; ++ci)
                for (int kd = 0; kd < 3; ++kd) {
                  if (!in_volume(xg, p + kd - 1)) continue;
                  for (int kh = 0; kh < 3; ++kh) {
                    const int64_t hh = h + kh - 1;
                    if (hh < 0 || hh >= H) continue;
                    for (int kw = 0; kw < 3; ++kw) {
                      const int64_t ww = v + kw - 1;
                      if (ww < 0 || ww >= W) continue;
                      acc += w[(((co * Ci + ci) * 3 + kd) * 3 + kh) * 3 + kw] * x[at5(xg, n, ci, p + kd - 1, hh, ww)];
                    }
                  }
                }
              if (!(acc > 0.0)) acc *= slope;
            }
            z[at5(zg, n, co, p, h, v)] = acc;
          }
      }
  return 0;
}

/* ------------------------------------------------------------ backward-data */
/* g = dz * (z > 0 ? 1 : slope)   (z = saved forward OUTPUT; NULL or ACT_NONE: g = dz)
 * dx[n,ci,q] = sum_{co,k} w[co,ci,k] * g~[n,co,q-k+1]
 * dx planes [-dx.halo_lo, d + dx.halo_hi); planes outside the volume are zero. */
int orc_conv3d_bwd_data(const double* dz, const int64_t* dzg, const double* z, const int64_t* zg,
                        const double* w, double* dx, const int64_t* dxg, int act, double alpha) {
  if (!same_shard(dzg, dxg)) return -1;
  const int masked = (z != NULL && act != ACT_NONE);
  if (masked && (!same_shard(zg, dzg) || zg[G_C] != dzg[G_C])) return -1;
  const int64_t N = dzg[G_N], Co = dzg[G_C], Ci = dxg[G_C], D = dzg[G_D], H = dzg[G_H], W = dzg[G_W];
  const int64_t qlo = -dxg[G_HLO], qhi = D + dxg[G_HHI];
  if (!halo_ok(dzg, qlo, qhi)) return -4;
  if (masked && !halo_ok(zg, qlo, qhi)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ci = 0; ci < Ci; ++ci)
      for (int64_t q = qlo; q < qhi; ++q) {
        const int inside = in_volume(dxg, q);
        for (int64_t h = 0; h < H; ++h)
          for (int64_t v = 0; v < W; ++v) {
            double acc = 0.0;
            if (inside)
              for (int64_t co = 0; co < Co; ++co)
                for (int kd = 0; kd < 3; ++kd) {
                  const int64_t p = q - kd + 1;
                  if (!in_volume(dzg, p)) continue;
                  for (int kh = 0; kh < 3; ++kh) {
                    const int64_t hh = h - kh + 1;
                    if (hh < 0 || hh >= H) continue;
                    for (int kw = 0; kw < 3; ++kw) {
                      const int64_t ww = v - kw + 1;
                      if (ww < 0 || ww >= W) continue;
                      double g = dz[at5(dzg, n, co, p, hh, ww)];
                      if (masked && !(z[at5(zg, n, co, p, hh, ww)] > 0.0)) g *= slope;
                      acc += w[(((co * Ci + ci) * 3 + kd) * 3 + kh) * 3 + kw] * g;
                    }
                  }
                }
            dx[at5(dxg, n, ci, q, h, v)] = acc;
          }
      }
  return 0;
}

/* ---------------------------------------------------------- backward-filter */
/* dw[co,ci,k] = sum_n sum_{p in shard interior} g[n,co,p] * x~[n,ci,p+k-1];
 * db[co] = sum g.  The shard's partial: summing the partials of all shards
 * gives the full gradient (the data-parallel/spatial allreduce of Sec. III-A). */
int orc_conv3d_bwd_filter(const double* x, const int64_t* xg, const double* dz, const int64_t* dzg,
                          const double* z, const int64_t* zg, double* dw, double* db, int act, double alpha) {
  if (!same_shard(xg, dzg)) return -1;
  const int masked = (z != NULL && act != ACT_NONE);
  if (masked && (!same_shard(zg, dzg) || zg[G_C] != dzg[G_C])) return -1;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = dzg[G_C], D = xg[G_D], H = xg[G_H], W = xg[G_W];
  if (!halo_ok(xg, 0, D)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t co = 0; co < Co; ++co)
    for (int64_t cik = 0; cik < Ci * 27; ++cik) {
      const int64_t ci = cik / 27;
      const int kd = (int)(cik % 27) / 9, kh = (int)(cik % 9) / 3, kw = (int)(cik % 3);
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < D; ++p) {
          if (!in_volume(xg, p + kd - 1)) continue;
          for (int64_t h = 0; h < H; ++h) {
            const int64_t hh = h + kh - 1;
            if (hh < 0 || hh >= H) continue;
            for (int64_t v = 0; v < W; ++v) {
              const int64_t ww = v + kw - 1;
              if (ww < 0 || ww >= W) continue;
              double g = dz[at5(dzg, n, co, p, h, v)];
              if (masked && !(z[at5(zg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g * x[at5(xg, n, ci, p + kd - 1, hh, ww)];
            }
          }
        }
      dw[co * Ci * 27 + cik] = acc;
    }
  if (db) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t co = 0; co < Co; ++co) {
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < D; ++p)
          for (int64_t h = 0; h < H; ++h)
            for (int64_t v = 0; v < W; ++v) {
              double g = dz[at5(dzg, n, co, p, h, v)];
              if (masked && !(z[at5(zg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g;
            }
      db[co] = acc;
    }
  }
  return 0;
}

/* ------------------------------------------------- 5x5x5 convolution */
/* Filters of 5x5x5 with stride 1 and two zero voxels of padding on every side (Sec. III-A names 3^3 and
 * 5^3 as the two filter sizes whose halo faces have specialised packing kernels; the halo is then two
 * planes wide).  Written for an odd filter edge K = 2R+1 so that K = 3 can be compared with the functions
 * above; the shard interior only is produced (no halo recompute):
 *   z[n,co,p]  = act(b[co] + sum_{ci,k} w[co,ci,k] * x~[n,ci,p+k-R])        p in [0,d)
 *   dx[n,ci,q] = sum_{co,k} w[co,ci,k] * g~[n,co,q-k+R],  g = dz * act'(z)   q in [0,d)
 *   dw[co,ci,k] = sum_{n,p in [0,d)} g[n,co,p] * x~[n,ci,p+k-R],  db[co] = sum g. */
static int halo_ok_r(const int64_t* in, int64_t R) {
  for (int64_t p = 0; p < in[G_D]; ++p)
    for (int64_t k = -R; k <= R; ++k)
      if (in_volume(in, p + k) && !stored(in, p + k)) return 0;
  return 1;
}

int orc_convk_fwd(int K, const double* x, const int64_t* xg, const double* w, const double* bias, double* z,
                  const int64_t* zg, int act, double alpha) {
  if (K < 1 || K % 2 == 0 || !same_shard(xg, zg)) return -1;
  const int64_t R = K / 2, N = xg[G_N], Ci = xg[G_C], Co = zg[G_C], D = xg[G_D], H = xg[G_H], W = xg[G_W];
  if (!halo_ok_r(xg, R)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t co = 0; co < Co; ++co)
      for (int64_t p = 0; p < D; ++p)
        for (int64_t h = 0; h < H; ++h)
          for (int64_t v = 0; v < W; ++v) {
            double acc = bias ? bias[co] : 0.0;
            for (int64_t ci = 0; ci < Ci; ++ci)
              for (int64_t kd = 0; kd < K; ++kd) {
                if (!in_volume(xg, p + kd - R)) continue;
                for (int64_t kh = 0; kh < K; ++kh) {
                  const int64_t hh = h + kh - R;
                  if (hh < 0 || hh >= H) continue;
                  for (int64_t kw = 0; kw < K; ++kw) {
                    const int64_t ww = v + kw - R;
                    if (ww < 0 || ww >= W) continue;
                    acc += w[(((co * Ci + ci) * K + kd) * K + kh) * K + kw] * x[at5(xg, n, ci, p + kd - R, hh, ww)];
                  }
                }
              }
            if (!(acc > 0.0)) acc *= slope;
            z[at5(zg, n, co, p, h, v)] = acc;
          }
  return 0;
}

int orc_convk_bwd_data(int K, const double* dz, const int64_t* dzg, const double* z, const int64_t* zg,
                       const double* w, double* dx, const int64_t* dxg, int act, double alpha) {
  if (K < 1 || K % 2 == 0 || !same_shard(dzg, dxg)) return -1;
  const int masked = (z != NULL && act != ACT_NONE);
  if (masked && (!same_shard(zg, dzg) || zg[G_C] != dzg[G_C])) return -1;
  const int64_t R = K / 2, N = dzg[G_N], Co = dzg[G_C], Ci = dxg[G_C], D = dzg[G_D], H = dzg[G_H], W = dzg[G_W];
  if (!halo_ok_r(dzg, R)) return -4;
  if (masked && !halo_ok_r(zg, R)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ci = 0; ci < Ci; ++ci)
      for (int64_t q = 0; q < D; ++q)
        for (int64_t h = 0; h < H; ++h)
          for (int64_t v = 0; v < W; ++v) {
            double acc = 0.0;
            for (int64_t co = 0; co < Co; ++co)
              for (int64_t kd = 0; kd < K; ++kd) {
                const int64_t p = q - kd + R;
                if (!in_volume(dzg, p)) continue;
                for (int64_t kh = 0; kh < K; ++kh) {
                  const int64_t hh = h - kh + R;
                  if (hh < 0 || hh >= H) continue;
                  for (int64_t kw = 0; kw < K; ++kw) {
                    const int64_t ww = v - kw + R;
                    if (ww < 0 || ww >= W) continue;
                    double g = dz[at5(dzg, n, co, p, hh, ww)];
                    if (masked && !(z[at5(zg, n, co, p, hh, ww)] > 0.0)) g *= slope;
                    acc += w[(((co * Ci + ci) * K + kd) * K + kh) * K + kw] * g;
                  }
                }
              }
            dx[at5(dxg, n, ci, q, h, v)] = acc;
          }
  return 0;
}

int orc_convk_bwd_filter(int K, const double* x, const int64_t* xg, const double* dz, const int64_t* dzg,
                         const double* z, const int64_t* zg, double* dw, double* db, int act, double alpha) {
  if (K < 1 || K % 2 == 0 || !same_shard(xg, dzg)) return -1;
  const int masked = (z != NULL && act != ACT_NONE);
  if (masked && (!same_shard(zg, dzg) || zg[G_C] != dzg[G_C])) return -1;
  const int64_t R = K / 2, K3 = (int64_t)K * K * K;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = dzg[G_C], D = xg[G_D], H = xg[G_H], W = xg[G_W];
  if (!halo_ok_r(xg, R)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t co = 0; co < Co; ++co)
    for (int64_t cik = 0; cik < Ci * K3; ++cik) {
      const int64_t ci = cik / K3, k = cik % K3;
      const int64_t kd = k / (K * K), kh = (k / K) % K, kw = k % K;
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < D; ++p) {
          if (!in_volume(xg, p + kd - R)) continue;
          for (int64_t h = 0; h < H; ++h) {
            const int64_t hh = h + kh - R;
            if (hh < 0 || hh >= H) continue;
            for (int64_t v = 0; v < W; ++v) {
              const int64_t ww = v + kw - R;
              if (ww < 0 || ww >= W) continue;
              double g = dz[at5(dzg, n, co, p, h, v)];
              if (masked && !(z[at5(zg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g * x[at5(xg, n, ci, p + kd - R, hh, ww)];
            }
          }
        }
      dw[co * Ci * K3 + cik] = acc;
    }
  if (db) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t co = 0; co < Co; ++co) {
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < D; ++p)
          for (int64_t h = 0; h < H; ++h)
            for (int64_t v = 0; v < W; ++v) {
              double g = dz[at5(dzg, n, co, p, h, v)];
              if (masked && !(z[at5(zg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g;
            }
      db[co] = acc;
    }
  }
  return 0;
}

/* ------------------------------------------------- stride-2 convolution */
/* The fourth convolution of the CosmoFlow network has a stride of 2 (Table I); "same" padding
 * is read as one zero voxel on every side, as for the stride-1 layers, so that an even extent is
 * halved (odd: rounded up):
 *   y[n,co,p] = act(b[co] + sum_{ci,k} w[co,ci,k] * x~[n,ci,2p+k-1]).
 * Slab form: x has even d, d_offset, d_global; y is the shard with all three halved and no halo
 * planes; output plane p reads input planes 2p-1..2p+1, so x needs its LOWER halo plane only. */
static int s2_shapes(const int64_t* xg, const int64_t* yg) {
  if (xg[G_D] % 2 || xg[G_DOFF] % 2 || xg[G_DGLOB] % 2) return 0;
  return yg[G_N] == xg[G_N] && yg[G_D] == xg[G_D] / 2 && yg[G_H] == (xg[G_H] + 1) / 2 && yg[G_W] == (xg[G_W] + 1) / 2 &&
         yg[G_DOFF] == xg[G_DOFF] / 2 && yg[G_DGLOB] == xg[G_DGLOB] / 2;
}

int orc_conv3d_s2_fwd(const double* x, const int64_t* xg, const double* w, const double* bias, double* y,
                      const int64_t* yg, int act, double alpha) {
  if (!s2_shapes(xg, yg) || yg[G_HLO] || yg[G_HHI]) return -1;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C], H = xg[G_H], W = xg[G_W];
  const int64_t Do = yg[G_D], Ho = yg[G_H], Wo = yg[G_W];
  if (Do > 0 && in_volume(xg, -1) && !stored(xg, -1)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t co = 0; co < Co; ++co)
      for (int64_t p = 0; p < Do; ++p)
        for (int64_t h = 0; h < Ho; ++h)
          for (int64_t v = 0; v < Wo; ++v) {
            double acc = bias ? bias[co] : 0.0;
            for (int64_t ci = 0; ci < Ci; ++ci)
              for (int kd = 0; kd < 3; ++kd) {
                const int64_t pp = 2 * p + kd - 1;
                if (!in_volume(xg, pp)) continue;
                for (int kh = 0; kh < 3; ++kh) {
                  const int64_t hh = 2 * h + kh - 1;
                  if (hh < 0 || hh >= H) continue;
                  for (int kw = 0; kw < 3; ++kw) {
                    const int64_t ww = 2 * v + kw - 1;
                    if (ww < 0 || ww >= W) continue;
                    acc += w[(((co * Ci + ci) * 3 + kd) * 3 + kh) * 3 + kw] * x[at5(xg, n, ci, pp, hh, ww)];
                  }
                }
              }
            if (!(acc > 0.0)) acc *= slope;
            y[at5(yg, n, co, p, h, v)] = acc;
          }
  return 0;
}

/* g = dy * (y > 0 ? 1 : slope);  dx[n,ci,q] = sum over (co,k,p) with 2p+k-1 = q of w[co,ci,k] * g[n,co,p]
 * for the interior planes q of the input shard.  Plane q = d-1 takes a term from output plane d/2, the
 * first plane of the shard above: dy (and y) need their UPPER halo plane when it is inside the volume. */
int orc_conv3d_s2_bwd_data(const double* dy, const int64_t* yg, const double* y, const int64_t* ysg, const double* w,
                           double* dx, const int64_t* xg, int act, double alpha) {
  if (!s2_shapes(xg, yg) || xg[G_HLO] || xg[G_HHI]) return -1;
  const int masked = (y != NULL && act != ACT_NONE);
  if (masked && (!same_shard(ysg, yg) || ysg[G_C] != yg[G_C])) return -1;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C], D = xg[G_D], H = xg[G_H], W = xg[G_W];
  const int64_t Do = yg[G_D], Ho = yg[G_H], Wo = yg[G_W];
  if (Do > 0 && in_volume(yg, Do) && (!stored(yg, Do) || (masked && !stored(ysg, Do)))) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ci = 0; ci < Ci; ++ci)
      for (int64_t q = 0; q < D; ++q)
        for (int64_t h = 0; h < H; ++h)
          for (int64_t v = 0; v < W; ++v) {
            double acc = 0.0;
            for (int64_t co = 0; co < Co; ++co)
              for (int kd = 0; kd < 3; ++kd) {
                const int64_t t = q + 1 - kd;            /* = 2p */
                if (t % 2 != 0 || !in_volume(yg, t / 2)) continue;
                for (int kh = 0; kh < 3; ++kh) {
                  const int64_t th = h + 1 - kh;
                  if (th % 2 != 0 || th < 0 || th / 2 >= Ho) continue;
                  for (int kw = 0; kw < 3; ++kw) {
                    const int64_t tw = v + 1 - kw;
                    if (tw % 2 != 0 || tw < 0 || tw / 2 >= Wo) continue;
                    double g = dy[at5(yg, n, co, t / 2, th / 2, tw / 2)];
                    if (masked && !(y[at5(ysg, n, co, t / 2, th / 2, tw / 2)] > 0.0)) g *= slope;
                    acc += w[(((co * Ci + ci) * 3 + kd) * 3 + kh) * 3 + kw] * g;
                  }
                }
              }
            dx[at5(xg, n, ci, q, h, v)] = acc;
          }
  return 0;
}

/* dw[co,ci,k] = sum_n sum_{p in the output shard} g[n,co,p] * x~[n,ci,2p+k-1]; db[co] = sum g: the shard's partial. */
int orc_conv3d_s2_bwd_filter(const double* x, const int64_t* xg, const double* dy, const int64_t* yg, const double* y,
                             const int64_t* ysg, double* dw, double* db, int act, double alpha) {
  if (!s2_shapes(xg, yg)) return -1;
  const int masked = (y != NULL && act != ACT_NONE);
  if (masked && (!same_shard(ysg, yg) || ysg[G_C] != yg[G_C])) return -1;
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C], H = xg[G_H], W = xg[G_W];
  const int64_t Do = yg[G_D], Ho = yg[G_H], Wo = yg[G_W];
  if (Do > 0 && in_volume(xg, -1) && !stored(xg, -1)) return -4;
  const double slope = act_slope(act, alpha);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t co = 0; co < Co; ++co)
    for (int64_t cik = 0; cik < Ci * 27; ++cik) {
      const int64_t ci = cik / 27;
      const int kd = (int)(cik % 27) / 9, kh = (int)(cik % 9) / 3, kw = (int)(cik % 3);
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < Do; ++p) {
          const int64_t pp = 2 * p + kd - 1;
          if (!in_volume(xg, pp)) continue;
          for (int64_t h = 0; h < Ho; ++h) {
            const int64_t hh = 2 * h + kh - 1;
            if (hh < 0 || hh >= H) continue;
            for (int64_t v = 0; v < Wo; ++v) {
              const int64_t ww = 2 * v + kw - 1;
              if (ww < 0 || ww >= W) continue;
              double g = dy[at5(yg, n, co, p, h, v)];
              if (masked && !(y[at5(ysg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g * x[at5(xg, n, ci, pp, hh, ww)];
            }
          }
        }
      dw[co * Ci * 27 + cik] = acc;
    }
  if (db) {
    for (int64_t co = 0; co < Co; ++co) {
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < Do; ++p)
          for (int64_t h = 0; h < Ho; ++h)
            for (int64_t v = 0; v < Wo; ++v) {
              double g = dy[at5(yg, n, co, p, h, v)];
              if (masked && !(y[at5(ysg, n, co, p, h, v)] > 0.0)) g *= slope;
              acc += g;
            }
      db[co] = acc;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------ pooling */
/* 2x2x2, stride 2, non-overlapping windows over the shard INTERIOR (Sec. III-A:
 * pooling is the other layer with a spatial dependency; with even d and even
 * d_offset no window straddles a shard face).  mode 0: average, mode 1: max.
 * y has interior extents d/2, h/2, w/2; halo planes of x and y are not touched. */
int orc_pool3d_fwd(const double* x, const int64_t* xg, double* y, const int64_t* yg, int mode) {
  if (xg[G_D] % 2 || xg[G_H] % 2 || xg[G_W] % 2 || xg[G_DOFF] % 2) return -1;
  if (yg[G_N] != xg[G_N] || yg[G_C] != xg[G_C] || yg[G_D] * 2 != xg[G_D] || yg[G_H] * 2 != xg[G_H] ||
      yg[G_W] * 2 != xg[G_W])
    return -1;
#pragma omp parallel for collapse(2)
  for (int64_t n = 0; n < yg[G_N]; ++n)
    for (int64_t c = 0; c < yg[G_C]; ++c)
      for (int64_t q = 0; q < yg[G_D]; ++q)
        for (int64_t h = 0; h < yg[G_H]; ++h)
          for (int64_t v = 0; v < yg[G_W]; ++v) {
            double s = 0.0, m = -INFINITY;
            for (int kd = 0; kd < 2; ++kd)
              for (int kh = 0; kh < 2; ++kh)
                for (int kw = 0; kw < 2; ++kw) {
                  double e = x[at5(xg, n, c, 2 * q + kd, 2 * h + kh, 2 * v + kw)];
                  s += e;
                  if (e > m) m = e;
                }
            y[at5(yg, n, c, q, h, v)] = mode == 0 ? s * 0.125 : m;
          }
  return 0;
}

/* avg: dx[2q+k] = dy[q]/8.  max: all of dy[q] goes to the FIRST maximal element
 * of the window in (kd,kh,kw) row-major order, zero to the others (x = the
 * forward input).  Only interior planes of dx are written. */
int orc_pool3d_bwd(const double* dy, const int64_t* yg, const double* x, const int64_t* xg, double* dx,
                   const int64_t* dxg, int mode) {
  if (dxg[G_D] % 2 || dxg[G_H] % 2 || dxg[G_W] % 2) return -1;
  if (yg[G_N] != dxg[G_N] || yg[G_C] != dxg[G_C] || yg[G_D] * 2 != dxg[G_D] || yg[G_H] * 2 != dxg[G_H] ||
      yg[G_W] * 2 != dxg[G_W])
    return -1;
  if (mode == 1 && x == NULL) return -1;
#pragma omp parallel for collapse(2)
  for (int64_t n = 0; n < yg[G_N]; ++n)
    for (int64_t c = 0; c < yg[G_C]; ++c)
      for (int64_t q = 0; q < yg[G_D]; ++q)
        for (int64_t h = 0; h < yg[G_H]; ++h)
          for (int64_t v = 0; v < yg[G_W]; ++v) {
            const double g = dy[at5(yg, n, c, q, h, v)];
            int best = 0;
            if (mode == 1) {
              double m = -INFINITY;
              for (int k = 0; k < 8; ++k) {
                double e = x[at5(xg, n, c, 2 * q + (k >> 2), 2 * h + ((k >> 1) & 1), 2 * v + (k & 1))];
                if (e > m) { m = e; best = k; }
              }
            }
            for (int k = 0; k < 8; ++k)
              dx[at5(dxg, n, c, 2 * q + (k >> 2), 2 * h + ((k >> 1) & 1), 2 * v + (k & 1))] =
                  mode == 0 ? g * 0.125 : (k == best ? g : 0.0);
          }
  return 0;
}

/* ------------------------------------------- 2x2x2 stride-2 transposed conv */
/* U-Net up-sampling (Sec. II-C, III-A "deconvolution").  Every output voxel
 * receives exactly one tap:  y[n,co,2q+k] = b[co] + sum_ci w[ci,co,k] * x[n,ci,q],
 * w laid out [cin][cout][2][2][2].  Interior planes only. */
int orc_deconv2_fwd(const double* x, const int64_t* xg, const double* w, const double* bias, double* y,
                    const int64_t* yg) {
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C];
  if (yg[G_D] != 2 * xg[G_D] || yg[G_H] != 2 * xg[G_H] || yg[G_W] != 2 * xg[G_W] || yg[G_N] != N) return -1;
#pragma omp parallel for collapse(3)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t co = 0; co < Co; ++co)
      for (int64_t p = 0; p < yg[G_D]; ++p)
        for (int64_t h = 0; h < yg[G_H]; ++h)
          for (int64_t v = 0; v < yg[G_W]; ++v) {
            const int k = (int)((p & 1) * 4 + (h & 1) * 2 + (v & 1));
            double acc = bias ? bias[co] : 0.0;
            for (int64_t ci = 0; ci < Ci; ++ci)
              acc += w[(ci * Co + co) * 8 + k] * x[at5(xg, n, ci, p / 2, h / 2, v / 2)];
            y[at5(yg, n, co, p, h, v)] = acc;
          }
  return 0;
}

/* dx[n,ci,q] = sum_{co,k} w[ci,co,k] * dy[n,co,2q+k] */
int orc_deconv2_bwd_data(const double* dy, const int64_t* yg, const double* w, double* dx, const int64_t* xg) {
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C];
  if (yg[G_D] != 2 * xg[G_D] || yg[G_H] != 2 * xg[G_H] || yg[G_W] != 2 * xg[G_W] || yg[G_N] != N) return -1;
#pragma omp parallel for collapse(3)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ci = 0; ci < Ci; ++ci)
      for (int64_t q = 0; q < xg[G_D]; ++q)
        for (int64_t h = 0; h < xg[G_H]; ++h)
          for (int64_t v = 0; v < xg[G_W]; ++v) {
            double acc = 0.0;
            for (int64_t co = 0; co < Co; ++co)
              for (int k = 0; k < 8; ++k)
                acc += w[(ci * Co + co) * 8 + k] *
                       dy[at5(yg, n, co, 2 * q + (k >> 2), 2 * h + ((k >> 1) & 1), 2 * v + (k & 1))];
            dx[at5(xg, n, ci, q, h, v)] = acc;
          }
  return 0;
}

/* dw[ci,co,k] = sum_{n,q} x[n,ci,q] * dy[n,co,2q+k];  db[co] = sum dy */
int orc_deconv2_bwd_filter(const double* x, const int64_t* xg, const double* dy, const int64_t* yg, double* dw,
                           double* db) {
  const int64_t N = xg[G_N], Ci = xg[G_C], Co = yg[G_C];
  if (yg[G_D] != 2 * xg[G_D] || yg[G_H] != 2 * xg[G_H] || yg[G_W] != 2 * xg[G_W] || yg[G_N] != N) return -1;
#pragma omp parallel for collapse(2)
  for (int64_t ci = 0; ci < Ci; ++ci)
    for (int64_t cok = 0; cok < Co * 8; ++cok) {
      const int64_t co = cok / 8;
      const int k = (int)(cok % 8);
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t q = 0; q < xg[G_D]; ++q)
          for (int64_t h = 0; h < xg[G_H]; ++h)
            for (int64_t v = 0; v < xg[G_W]; ++v)
              acc += x[at5(xg, n, ci, q, h, v)] *
                     dy[at5(yg, n, co, 2 * q + (k >> 2), 2 * h + ((k >> 1) & 1), 2 * v + (k & 1))];
      dw[ci * Co * 8 + cok] = acc;
    }
  if (db)
    for (int64_t co = 0; co < Co; ++co) {
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < yg[G_D]; ++p)
          for (int64_t h = 0; h < yg[G_H]; ++h)
            for (int64_t v = 0; v < yg[G_W]; ++v) acc += dy[at5(yg, n, co, p, h, v)];
      db[co] = acc;
    }
  return 0;
}

int orc_num_threads(void) {
  int t = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    t = omp_get_num_threads();
  }
#endif
  return t;
}
