// 2x2x2 stride-2 average / max pooling of a slab interior, forward and backward.
// Pure streaming kernels (HBM-bound: 8 elements read per element written, or the reverse):
// each thread produces VEC consecutive outputs along W from four input rows read with 16-byte
// loads, so a wavefront covers whole 128-byte lines of every row it touches.
#include "common.h"

namespace h3d {

template <typename T, int N>
struct alignas(sizeof(T) * N) Vec {
  T v[N];
};

struct PoolArgs {
  Geo x, y;            // x: the big tensor (fwd input / bwd output), y: the pooled one
  int64_t total;       // threads needed = n*c*yd*yh*(yw/VEC)
  int wv;              // yw / VEC
};

template <typename T, int VEC>
__device__ __forceinline__ void decode(const PoolArgs& a, int64_t t, int64_t& xoff, int64_t& yoff) {
  int wv = (int)(t % a.wv); t /= a.wv;
  int ho = (int)(t % a.y.h); t /= a.y.h;
  int q = (int)(t % a.y.d); t /= a.y.d;
  int c = (int)(t % a.y.c);
  int n = (int)(t / a.y.c);
  yoff = n * a.y.nstride + c * a.y.cstride + (int64_t)(q + a.y.hlo) * a.y.plane + (int64_t)ho * a.y.w + wv * VEC;
  xoff = n * a.x.nstride + c * a.x.cstride + (int64_t)(2 * q + a.x.hlo) * a.x.plane + (int64_t)(2 * ho) * a.x.w +
         wv * VEC * 2;
}

template <typename T, int VEC, int MODE>
__global__ void __launch_bounds__(256) pool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, PoolArgs a) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int64_t xoff, yoff;
  decode<T, VEC>(a, t, xoff, yoff);
  Vec<T, 2 * VEC> r[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    r[k] = *reinterpret_cast<const Vec<T, 2 * VEC>*>(x + xoff + (k >> 1) * a.x.plane + (k & 1) * a.x.w);
  Vec<T, VEC> o;
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    if (MODE == H3D_POOL_AVG) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) s += ld(&r[k].v[2 * i]) + ld(&r[k].v[2 * i + 1]);
      st(&o.v[i], s * 0.125f);
    } else {
      T best = r[0].v[2 * i];
      float m = ld(&best);
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float e = ld(&r[k].v[2 * i + j]);
          if (e > m) { m = e; best = r[k].v[2 * i + j]; }
        }
      o.v[i] = best;
    }
  }
  *reinterpret_cast<Vec<T, VEC>*>(y + yoff) = o;
}

// Average pooling that also writes the sign mask of its input (bf16, 8 outputs = 16 inputs per thread and row): the
// activation output is read here anyway, so the backward pass can take the 1-bit mask instead of reading it again.
// Same pooled bits as pool_fwd_kernel<bf16_t, 8, AVG>, same mask bits as act_mask_kernel.
__global__ void __launch_bounds__(256) pool_fwd_mask_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                                                            uint8_t* __restrict__ mask, PoolArgs a) {
  constexpr int VEC = 8;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int64_t xoff, yoff;
  decode<bf16_t, VEC>(a, t, xoff, yoff);
  int64_t r0 = t;
  const int wv = (int)(r0 % a.wv); r0 /= a.wv;
  const int ho = (int)(r0 % a.y.h); r0 /= a.y.h;
  const int q = (int)(r0 % a.y.d); r0 /= a.y.d;          // r0 = n * c + channel
  Vec<bf16_t, 2 * VEC> r[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    r[k] = *reinterpret_cast<const Vec<bf16_t, 2 * VEC>*>(x + xoff + (k >> 1) * a.x.plane + (k & 1) * a.x.w);
  Vec<bf16_t, VEC> o;
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) s += ld(&r[k].v[2 * i]) + ld(&r[k].v[2 * i + 1]);
    st(&o.v[i], s * 0.125f);
  }
  *reinterpret_cast<Vec<bf16_t, VEC>*>(y + yoff) = o;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    uint32_t bits = 0;
#pragma unroll
    for (int e = 0; e < 2 * VEC; ++e) bits |= ((int16_t)r[k].v[e] > 0 ? 1u : 0u) << e;     // a bf16 is > 0 iff its bits, as int16, are
    const int64_t row = ((r0 * a.x.d + 2 * q + (k >> 1)) * a.x.h + 2 * ho + (k & 1)) * (a.x.w / 8) + 2 * wv;
    *reinterpret_cast<uint16_t*>(mask + row) = (uint16_t)bits;
  }
}

// ACT: also multiply by the activation derivative taken from the saved output z of the layer that
// produced the pooled tensor (g = pool_bwd(dy) * (z > 0 ? 1 : slope)): one pass instead of a pooling
// backward followed by an activation backward.
// ADD: a second gradient of the big tensor's shape (the skip branch of a U-Net level) is added to the un-pooled one
// before the activation derivative: g = (pool_bwd(dy) + dz2) * (z > 0 ? 1 : slope), rounded once.
template <typename T, int VEC, int MODE, bool ACT, bool ADD>
__global__ void __launch_bounds__(256) pool_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                       T* __restrict__ dx, PoolArgs a, Geo xin, const T* __restrict__ z,
                                                       Geo zg, float slope, const T* __restrict__ dz2, Geo d2g) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int64_t dxoff, yoff;
  decode<T, VEC>(a, t, dxoff, yoff);
  Vec<T, VEC> g = *reinterpret_cast<const Vec<T, VEC>*>(dy + yoff);
  Vec<T, 2 * VEC> o[4];
  Vec<T, 2 * VEC> r[4];          // rows of the pooling's forward input (max pooling)
  // a ReLU'd tensor that was max-pooled is both the pooling's input and the saved activation: read it once
  const bool z_is_x = MODE == H3D_POOL_MAX && ACT && z == x && zg.cstride == xin.cstride && zg.nstride == xin.nstride && zg.hlo == xin.hlo;
  if (MODE == H3D_POOL_AVG) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      T v;
      st(&v, ld(&g.v[i]) * 0.125f);
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k].v[2 * i] = o[k].v[2 * i + 1] = v;
    }
  } else {
    // same (n,c,q,ho,wv) decode against the forward input's own geometry (its halos may differ)
    PoolArgs b = a;
    b.x = xin;
    int64_t xoff, dummy;
    decode<T, VEC>(b, t, xoff, dummy);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      r[k] = *reinterpret_cast<const Vec<T, 2 * VEC>*>(x + xoff + (k >> 1) * xin.plane + (k & 1) * xin.w);
    T zero;
    st(&zero, 0.f);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float m = ld(&r[0].v[2 * i]);
      int best = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float e = ld(&r[k].v[2 * i + j]);
          if (e > m) { m = e; best = k * 2 + j; }   // strict: ties keep the first in (kd,kh,kw) order
        }
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < 2; ++j) o[k].v[2 * i + j] = (best == k * 2 + j) ? g.v[i] : zero;
    }
  }
  if (ACT || ADD) {
    PoolArgs b = a;
    b.x = zg;
    int64_t zoff = 0, d2off = 0, dummy;
    if (ACT) decode<T, VEC>(b, t, zoff, dummy);
    b.x = d2g;
    if (ADD) decode<T, VEC>(b, t, d2off, dummy);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      Vec<T, 2 * VEC> m, e;
      if (ACT) {
        if (z_is_x) m = r[k];
        else m = *reinterpret_cast<const Vec<T, 2 * VEC>*>(z + zoff + (k >> 1) * zg.plane + (k & 1) * zg.w);
      }
      if (ADD) e = *reinterpret_cast<const Vec<T, 2 * VEC>*>(dz2 + d2off + (k >> 1) * d2g.plane + (k & 1) * d2g.w);
#pragma unroll
      for (int i = 0; i < 2 * VEC; ++i) {
        if (ADD) {
          float v = ld(&o[k].v[i]) + ld(&e.v[i]);
          if (ACT && !(ld(&m.v[i]) > 0.f)) v *= slope;
          st(&o[k].v[i], v);
        } else if (!(ld(&m.v[i]) > 0.f)) {
          st(&o[k].v[i], ld(&o[k].v[i]) * slope);
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k)
    *reinterpret_cast<Vec<T, 2 * VEC>*>(dx + dxoff + (k >> 1) * a.x.plane + (k & 1) * a.x.w) = o[k];
}

// Sign mask of a saved activation output: bit k of byte j of a row = (z[8 j + k] > 0); rows packed
// [n][c][interior plane][h][w/8].  One thread per byte.
template <typename T>
__global__ void __launch_bounds__(256) act_mask_kernel(const T* __restrict__ z, uint8_t* __restrict__ mask, Geo g, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int64_t t = i;
  const int wb = (int)(t % (g.w / 8)); t /= g.w / 8;
  const int h = (int)(t % g.h); t /= g.h;
  const int p = (int)(t % g.d); t /= g.d;
  const int c = (int)(t % g.c);
  const int64_t n = t / g.c;
  const T* src = z + n * g.nstride + c * g.cstride + (int64_t)(p + g.hlo) * g.plane + (int64_t)h * g.w + 8 * wb;
  uint32_t bits = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) bits |= (ld(src + k) > 0.f ? 1u : 0u) << k;
  mask[i] = (uint8_t)bits;
}

// Average-pooling backward fused with the activation derivative read from the sign mask instead of the saved
// output: g = dy / 8 (rounded to storage) where the bit is set, that value times slope (rounded again) elsewhere —
// bit for bit what pool_bwd_kernel<.., ACT> writes from z itself, for 1/16 of its mask traffic.
__global__ void __launch_bounds__(256) pool_bwd_mask_kernel(const bf16_t* __restrict__ dy, const uint8_t* __restrict__ mask,
                                                            bf16_t* __restrict__ g, PoolArgs a, float slope) {
  constexpr int VEC = 8;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int64_t goff, yoff;
  decode<bf16_t, VEC>(a, t, goff, yoff);
  int64_t r = t;
  const int wv = (int)(r % a.wv); r /= a.wv;
  const int ho = (int)(r % a.y.h); r /= a.y.h;
  const int q = (int)(r % a.y.d); r /= a.y.d;      // r = n * C + c
  const Vec<bf16_t, VEC> gy = *reinterpret_cast<const Vec<bf16_t, VEC>*>(dy + yoff);
  bf16_t v[VEC], vs[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    v[i] = f32_to_bf16(bf16_to_f32(gy.v[i]) * 0.125f);
    vs[i] = f32_to_bf16(bf16_to_f32(v[i]) * slope);
  }
  const int64_t mrow = ((r * a.x.d + 2 * q) * a.x.h + 2 * ho) * (a.x.w / 8) + 2 * wv;   // byte of the first of the four rows
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t m = *reinterpret_cast<const uint16_t*>(mask + mrow + ((int64_t)(k >> 1) * a.x.h + (k & 1)) * (a.x.w / 8));
    Vec<bf16_t, 2 * VEC> o;
#pragma unroll
    for (int i = 0; i < 2 * VEC; ++i) o.v[i] = ((m >> i) & 1u) ? v[i >> 1] : vs[i >> 1];
    *reinterpret_cast<Vec<bf16_t, 2 * VEC>*>(g + goff + (k >> 1) * a.x.plane + (k & 1) * a.x.w) = o;
  }
}

static h3d_status pool_check(void* handle, const h3d_tensor* big, const h3d_tensor* small, const char* what) {
  if (big->dtype != small->dtype || big->n != small->n || big->c != small->c)
    return fail(handle, H3D_EINVAL, "%s: n/c/dtype mismatch", what);
  if ((big->d & 1) || (big->h & 1) || (big->w & 1) || (big->d_offset & 1) || (big->d_global & 1))
    return fail(handle, H3D_EUNSUPPORTED, "%s: d,h,w,d_offset,d_global must be even (a window would straddle a face)", what);
  if (small->d * 2 != big->d || small->h * 2 != big->h || small->w * 2 != big->w ||
      small->d_offset * 2 != big->d_offset || small->d_global * 2 != big->d_global)
    return fail(handle, H3D_EINVAL, "%s: pooled extents/offsets must be half of the input's", what);
  return H3D_OK;
}

h3d_status pool_shapes_check(void* handle, const h3d_tensor* big, const h3d_tensor* small, const char* what) {
  return pool_check(handle, big, small, what);
}

template <typename T>
static int pick_vec(const h3d_tensor* big, const h3d_tensor* small, const h3d_tensor* extra, const h3d_tensor* extra2 = nullptr,
                    const h3d_tensor* extra3 = nullptr) {
  // widest VEC (outputs per thread) such that every row start is aligned for the vector accesses
  const int cand = 16 / (2 * (int)sizeof(T)) * 2;  // bf16: 8, fp32: 4  (two 16-byte loads per input row)
  for (int v = cand; v > 1; v >>= 1) {
    bool ok = small->w % v == 0 && ((uintptr_t)small->data % (v * sizeof(T))) == 0 &&
              ((uintptr_t)big->data % (2 * v * sizeof(T))) == 0 &&
              (!extra || ((uintptr_t)extra->data % (2 * v * sizeof(T))) == 0) &&
              (!extra2 || ((uintptr_t)extra2->data % (2 * v * sizeof(T))) == 0) &&
              (!extra3 || ((uintptr_t)extra3->data % (2 * v * sizeof(T))) == 0);
    if (ok) return v;
  }
  return 0;  // scalar: VEC = 1 needs pairs aligned to 2 elements
}

template <typename T, int MODE>
static h3d_status pool_launch(void* handle, bool fwd, const h3d_tensor* big, const h3d_tensor* small,
                              const h3d_tensor* xin, hipStream_t stream, const h3d_tensor* zt = nullptr, float slope = 1.f,
                              const h3d_tensor* d2t = nullptr) {
  PoolArgs a;
  a.x = make_geo(big);
  a.y = make_geo(small);
  int vec = pick_vec<T>(big, small, xin, zt, d2t);
  if (vec == 0) {
    bool ok = ((uintptr_t)big->data % (2 * sizeof(T))) == 0 && (!xin || ((uintptr_t)xin->data % (2 * sizeof(T))) == 0) &&
              (!zt || ((uintptr_t)zt->data % (2 * sizeof(T))) == 0) && (!d2t || ((uintptr_t)d2t->data % (2 * sizeof(T))) == 0);
    if (!ok) return fail(handle, H3D_EUNSUPPORTED, "pool3d: data pointers must be aligned to two elements");
    vec = 1;
  }
  a.wv = small->w / vec;
  a.total = (int64_t)small->n * small->c * small->d * small->h * a.wv;
  if (a.total == 0) return H3D_OK;
  int64_t grid = cdiv(a.total, 256);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "pool3d: too many blocks");
  Geo gx = xin ? make_geo(xin) : a.x;
  Geo gz = zt ? make_geo(zt) : a.x;
  Geo gd2 = d2t ? make_geo(d2t) : a.x;
  const T* zp = zt ? (const T*)zt->data : nullptr;
  const T* d2p = d2t ? (const T*)d2t->data : nullptr;
  const T* bigp = (const T*)big->data;
  const T* smallp = (const T*)small->data;
#define H3D_POOL_CASE(V)                                                                                           \
  case V:                                                                                                          \
    if (fwd)                                                                                                       \
      hipLaunchKernelGGL((pool_fwd_kernel<T, V, MODE>), dim3((unsigned)grid), dim3(256), 0, stream, bigp,          \
                         (T*)small->data, a);                                                                      \
    else if (zt && d2t)                                                                                            \
      hipLaunchKernelGGL((pool_bwd_kernel<T, V, MODE, true, true>), dim3((unsigned)grid), dim3(256), 0, stream,    \
                         smallp, xin ? (const T*)xin->data : nullptr, (T*)big->data, a, gx, zp, gz, slope, d2p, gd2); \
    else if (zt)                                                                                                   \
      hipLaunchKernelGGL((pool_bwd_kernel<T, V, MODE, true, false>), dim3((unsigned)grid), dim3(256), 0, stream,   \
                         smallp, xin ? (const T*)xin->data : nullptr, (T*)big->data, a, gx, zp, gz, slope, d2p, gd2); \
    else if (d2t)                                                                                                  \
      hipLaunchKernelGGL((pool_bwd_kernel<T, V, MODE, false, true>), dim3((unsigned)grid), dim3(256), 0, stream,   \
                         smallp, xin ? (const T*)xin->data : nullptr, (T*)big->data, a, gx, zp, gz, slope, d2p, gd2); \
    else                                                                                                           \
      hipLaunchKernelGGL((pool_bwd_kernel<T, V, MODE, false, false>), dim3((unsigned)grid), dim3(256), 0, stream,  \
                         smallp, xin ? (const T*)xin->data : nullptr, (T*)big->data, a, gx, zp, gz, slope, d2p, gd2); \
    break;
  switch (vec) {
    H3D_POOL_CASE(8)
    H3D_POOL_CASE(4)
    H3D_POOL_CASE(2)
    H3D_POOL_CASE(1)
  }
#undef H3D_POOL_CASE
  return launch_status(handle, fwd ? "pool3d_fwd" : "pool3d_bwd");
}

}  // namespace h3d

using namespace h3d;

extern "C" h3d_status h3d_pool3d_fwd(void* handle, const h3d_tensor* x, h3d_tensor* y, int mode, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor(handle, x, "x"));
  H3D_TRY(check_tensor(handle, y, "y"));
  if (mode != H3D_POOL_AVG && mode != H3D_POOL_MAX) return fail(handle, H3D_EINVAL, "pool3d_fwd: bad mode %d", mode);
  H3D_TRY(pool_check(handle, x, y, "pool3d_fwd"));
  hipStream_t s = (hipStream_t)stream;
  if (x->dtype == H3D_F32)
    return mode == H3D_POOL_AVG ? pool_launch<float, H3D_POOL_AVG>(handle, true, x, y, nullptr, s)
                                : pool_launch<float, H3D_POOL_MAX>(handle, true, x, y, nullptr, s);
  return mode == H3D_POOL_AVG ? pool_launch<bf16_t, H3D_POOL_AVG>(handle, true, x, y, nullptr, s)
                              : pool_launch<bf16_t, H3D_POOL_MAX>(handle, true, x, y, nullptr, s);
}

static h3d_status pool_bwd_impl(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const h3d_tensor* z, const h3d_tensor* dz2,
                                h3d_tensor* dx, int mode, float slope, void* stream);

extern "C" h3d_status h3d_pool3d_bwd(void* handle, const h3d_tensor* dy, const h3d_tensor* x, h3d_tensor* dx, int mode,
                                     void* stream) {
  return pool_bwd_impl(handle, dy, x, nullptr, nullptr, dx, mode, 1.f, stream);
}

extern "C" h3d_status h3d_pool3d_bwd_act(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const h3d_tensor* z,
                                         const h3d_tensor* dz2, h3d_tensor* g, int mode, int act, float alpha, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "pool3d_bwd_act: bad activation");
  if (act == H3D_ACT_NONE) z = nullptr;
  else if (!z) return fail(handle, H3D_EINVAL, "pool3d_bwd_act: the saved output z is required");
  return pool_bwd_impl(handle, dy, x, z, dz2, g, mode, act_slope(act, alpha), stream);
}

static h3d_status pool_bwd_impl(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const h3d_tensor* z, const h3d_tensor* dz2,
                                h3d_tensor* dx, int mode, float slope, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (z) {
    H3D_TRY(check_tensor(handle, z, "z"));
    if (!dx || !same_shard(z, dx) || z->c != dx->c) return fail(handle, H3D_EINVAL, "pool3d_bwd_act: z and g shapes differ");
  }
  if (dz2) {
    H3D_TRY(check_tensor(handle, dz2, "dz2"));
    if (!dx || !same_shard(dz2, dx) || dz2->c != dx->c) return fail(handle, H3D_EINVAL, "pool3d_bwd_act: dz2 and g shapes differ");
  }
  H3D_TRY(check_tensor(handle, dy, "dy"));
  H3D_TRY(check_tensor(handle, dx, "dx"));
  if (mode != H3D_POOL_AVG && mode != H3D_POOL_MAX) return fail(handle, H3D_EINVAL, "pool3d_bwd: bad mode %d", mode);
  H3D_TRY(pool_check(handle, dx, dy, "pool3d_bwd"));
  if (mode == H3D_POOL_MAX) {
    if (!x) return fail(handle, H3D_EINVAL, "pool3d_bwd: max pooling needs the forward input x");
    H3D_TRY(check_tensor(handle, x, "x"));
    if (!same_shard(x, dx) || x->c != dx->c) return fail(handle, H3D_EINVAL, "pool3d_bwd: x and dx shapes differ");
  } else {
    x = nullptr;
  }
  hipStream_t s = (hipStream_t)stream;
  if (dx->dtype == H3D_F32)
    return mode == H3D_POOL_AVG ? pool_launch<float, H3D_POOL_AVG>(handle, false, dx, dy, x, s, z, slope, dz2)
                                : pool_launch<float, H3D_POOL_MAX>(handle, false, dx, dy, x, s, z, slope, dz2);
  return mode == H3D_POOL_AVG ? pool_launch<bf16_t, H3D_POOL_AVG>(handle, false, dx, dy, x, s, z, slope, dz2)
                              : pool_launch<bf16_t, H3D_POOL_MAX>(handle, false, dx, dy, x, s, z, slope, dz2);
}

extern "C" size_t h3d_act_mask_bytes(const h3d_tensor* z) {
  if (!z || z->w % 8 || z->n <= 0 || z->c <= 0 || z->d <= 0 || z->h <= 0) return 0;
  return (size_t)z->n * z->c * z->d * z->h * (z->w / 8);
}

extern "C" h3d_status h3d_act_mask(void* handle, const h3d_tensor* z, void* mask, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor_packed(handle, z, "z"));
  if (z->w % 8) return fail(handle, H3D_EUNSUPPORTED, "act_mask: w must be a multiple of 8");
  const int64_t total = (int64_t)h3d_act_mask_bytes(z);
  if (total == 0) return H3D_OK;
  if (!mask) return fail(handle, H3D_EINVAL, "act_mask: NULL mask");
  const Geo g = make_geo(z);
  const int64_t grid = cdiv(total, 256);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "act_mask: too many blocks");
  if (z->dtype == H3D_F32)
    hipLaunchKernelGGL((act_mask_kernel<float>), dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, (const float*)z->data, (uint8_t*)mask, g, total);
  else
    hipLaunchKernelGGL((act_mask_kernel<bf16_t>), dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, (const bf16_t*)z->data, (uint8_t*)mask, g, total);
  return launch_status(handle, "act_mask");
}

extern "C" h3d_status h3d_pool3d_fwd_mask(void* handle, const h3d_tensor* x, h3d_tensor* y, void* mask, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor_packed(handle, x, "x"));
  H3D_TRY(check_tensor_packed(handle, y, "y"));
  H3D_TRY(pool_check(handle, x, y, "pool3d_fwd_mask"));
  if (x->dtype != H3D_BF16 || x->w % 16 || (uintptr_t)x->data % 32 || (uintptr_t)y->data % 16 || (uintptr_t)mask % 2)
    return fail(handle, H3D_EUNSUPPORTED, "pool3d_fwd_mask: bf16, w a multiple of 16 and aligned tensors only");
  PoolArgs a;
  a.x = make_geo(x);
  a.y = make_geo(y);
  a.wv = y->w / 8;
  a.total = (int64_t)y->n * y->c * y->d * y->h * a.wv;
  if (a.total == 0) return H3D_OK;
  if (!mask) return fail(handle, H3D_EINVAL, "pool3d_fwd_mask: NULL mask");
  const int64_t grid = cdiv(a.total, 256);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "pool3d_fwd_mask: too many blocks");
  hipLaunchKernelGGL(pool_fwd_mask_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, (const bf16_t*)x->data,
                     (bf16_t*)y->data, (uint8_t*)mask, a);
  return launch_status(handle, "pool3d_fwd_mask");
}

extern "C" h3d_status h3d_pool3d_bwd_mask(void* handle, const h3d_tensor* dy, const void* mask, h3d_tensor* g, int act, float alpha,
                                          void* stream) {
  if (!handle) return H3D_EINVAL;
  if (act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "pool3d_bwd_mask: activation must be RELU or LEAKY");
  H3D_TRY(check_tensor_packed(handle, dy, "dy"));
  H3D_TRY(check_tensor_packed(handle, g, "g"));
  H3D_TRY(pool_check(handle, g, dy, "pool3d_bwd_mask"));
  if (g->dtype != H3D_BF16 || g->w % 16 || (uintptr_t)g->data % 32 || (uintptr_t)dy->data % 16 || (uintptr_t)mask % 2)
    return fail(handle, H3D_EUNSUPPORTED, "pool3d_bwd_mask: bf16, w a multiple of 16 and aligned tensors only");
  PoolArgs a;
  a.x = make_geo(g);
  a.y = make_geo(dy);
  a.wv = dy->w / 8;
  a.total = (int64_t)dy->n * dy->c * dy->d * dy->h * a.wv;
  if (a.total == 0) return H3D_OK;
  if (!mask) return fail(handle, H3D_EINVAL, "pool3d_bwd_mask: NULL mask");
  const int64_t grid = cdiv(a.total, 256);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "pool3d_bwd_mask: too many blocks");
  hipLaunchKernelGGL(pool_bwd_mask_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, (const bf16_t*)dy->data,
                     (const uint8_t*)mask, (bf16_t*)g->data, a, act_slope(act, alpha));
  return launch_status(handle, "pool3d_bwd_mask");
}
