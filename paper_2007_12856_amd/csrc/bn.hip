// Local parts of distributed batch normalisation (Sec. II-B: partial statistics per shard, allreduce, per-channel
// affine map; Sec. III-C: its cost = this computation + the allreduce of the per-channel sum and squared sum).
// All four passes are HBM-bound streams over the interior planes of a slab (a contiguous run per sample and
// channel): 16-byte loads, fp32 arithmetic.  The reductions are deterministic: every (sample, channel) run is cut
// into segments by shape alone, a block sums one segment in a fixed order, and a second kernel adds the
// segments of a channel in order (in fp64) — no atomics.
#include <algorithm>

#include "common.h"

namespace h3d {
namespace {

constexpr int BN_SEG = 131072;       // elements of one (sample, channel) run summed by one block

struct BnArgs {
  Geo x, y;            // y: second tensor of the pass (dy, or the output)
  int segs;            // segments per (sample, channel) run
  int64_t run;         // d * h * w
};

template <typename T, int V> struct alignas(V * sizeof(T)) BnPack { T v[V]; };

// block-wide sum of two values in a fixed order: lanes by butterfly, wavefronts in index order
__device__ __forceinline__ void bn_block_sum2(float& a, float& b) {
  __shared__ float red[2][4];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) { a += __shfl_xor(a, off, 64); b += __shfl_xor(b, off, 64); }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) { red[0][wave] = a; red[1][wave] = b; }
  __syncthreads();
  a = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
  b = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
}

// MODE 0: (sum x, sum x^2).  MODE 1: (sum dy, sum dy * (x - mean) * invstd) with y = dy.
// part: [c][n * segs][2]
template <typename T, int MODE>
__global__ void __launch_bounds__(256) bn_partial_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                         const float* __restrict__ mean, const float* __restrict__ invstd,
                                                         float* __restrict__ part, BnArgs a) {
  constexpr int V = 16 / sizeof(T);
  const int seg = blockIdx.x, c = blockIdx.y, n = blockIdx.z;
  const int64_t e0 = (int64_t)seg * BN_SEG, e1 = min(e0 + BN_SEG, a.run);
  const T* xp = x + n * a.x.nstride + c * a.x.cstride + (int64_t)a.x.hlo * a.x.plane;
  const T* gp = MODE == 1 ? dy + n * a.y.nstride + c * a.y.cstride + (int64_t)a.y.hlo * a.y.plane : nullptr;
  const float mu = MODE == 1 ? mean[c] : 0.f, is = MODE == 1 ? invstd[c] : 0.f;
  float s0 = 0.f, s1 = 0.f;
  const bool vec = (uintptr_t)xp % 16 == 0 && (MODE == 0 || (uintptr_t)gp % 16 == 0);
  if (vec) {
    // four 16-byte loads in flight per thread and tensor
    constexpr int UN = 4;
    for (int64_t eb = e0 + (int64_t)threadIdx.x * V; eb < e1; eb += (int64_t)256 * V * UN) {
      BnPack<T, V> px[UN], pg[MODE == 1 ? UN : 1];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int64_t e = eb + (int64_t)u * 256 * V;
        if (e + V <= e1) {
          px[u] = *reinterpret_cast<const BnPack<T, V>*>(xp + e);
          if (MODE == 1) pg[u] = *reinterpret_cast<const BnPack<T, V>*>(gp + e);
        }
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int64_t e = eb + (int64_t)u * 256 * V;
        if (e + V <= e1) {
          if (MODE == 0) {
#pragma unroll
            for (int i = 0; i < V; ++i) { const float v = ld(&px[u].v[i]); s0 += v; s1 = fmaf(v, v, s1); }
          } else {
#pragma unroll
            for (int i = 0; i < V; ++i) { const float g = ld(&pg[u].v[i]); s0 += g; s1 = fmaf(g, (ld(&px[u].v[i]) - mu) * is, s1); }
          }
        }
      }
    }
    // the segment's ragged tail (fewer than V elements): thread 0
    const int64_t tail = e0 + (e1 - e0) / V * V;
    if (threadIdx.x == 0)
      for (int64_t e = tail; e < e1; ++e) {
        const float v = ld(xp + e);
        if (MODE == 0) { s0 += v; s1 = fmaf(v, v, s1); }
        else { const float g = ld(gp + e); s0 += g; s1 = fmaf(g, (v - mu) * is, s1); }
      }
  } else {
    for (int64_t e = e0 + threadIdx.x; e < e1; e += 256) {
      const float v = ld(xp + e);
      if (MODE == 0) { s0 += v; s1 = fmaf(v, v, s1); }
      else { const float g = ld(gp + e); s0 += g; s1 = fmaf(g, (v - mu) * is, s1); }
    }
  }
  bn_block_sum2(s0, s1);
  if (threadIdx.x == 0) {
    float* o = part + (((int64_t)c * gridDim.z + n) * a.segs + seg) * 2;
    o[0] = s0; o[1] = s1;
  }
}

__global__ void bn_reduce_kernel(const float* __restrict__ part, float* __restrict__ out0, float* __restrict__ out1, int c, int per) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  double s0 = 0.0, s1 = 0.0;
  const float* p = part + (int64_t)ch * per * 2;
  for (int i = 0; i < per; ++i) { s0 += p[2 * i]; s1 += p[2 * i + 1]; }
  out0[ch] = (float)s0; out1[ch] = (float)s1;
}

// y = x * sc[c] + sh[c] (forward), or dx = dy * k1[c] + x * k2[c] + k3[c] (backward): coefficient tables in `coef`
// coef: [c][4] = {a, b, c, unused};  out = in0 * a + in1 * b + c   (in1 unused when b == 0 and TWO == false)
template <typename T, bool TWO>
__global__ void __launch_bounds__(256) bn_apply_kernel(const T* __restrict__ in0, const T* __restrict__ in1, T* __restrict__ out,
                                                       const float* __restrict__ coef, Geo g0, Geo g1, Geo go, int64_t run) {
  constexpr int V = 16 / sizeof(T);
  const int c = blockIdx.y, n = blockIdx.z;
  const float ka = coef[4 * c], kb = coef[4 * c + 1], kc = coef[4 * c + 2];
  const T* p0 = in0 + n * g0.nstride + c * g0.cstride + (int64_t)g0.hlo * g0.plane;
  const T* p1 = TWO ? in1 + n * g1.nstride + c * g1.cstride + (int64_t)g1.hlo * g1.plane : nullptr;
  T* po = out + n * go.nstride + c * go.cstride + (int64_t)go.hlo * go.plane;
  const bool vec = (uintptr_t)p0 % 16 == 0 && (uintptr_t)po % 16 == 0 && (!TWO || (uintptr_t)p1 % 16 == 0);
  const int64_t stride = (int64_t)gridDim.x * 256;
  if (vec) {
    const int64_t nv = run / V;
    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < nv; u += stride) {
      const BnPack<T, V> a = *reinterpret_cast<const BnPack<T, V>*>(p0 + u * V);
      BnPack<T, V> b, o;
      if (TWO) b = *reinterpret_cast<const BnPack<T, V>*>(p1 + u * V);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        float r = fmaf(ld(&a.v[i]), ka, kc);
        if (TWO) r = fmaf(ld(&b.v[i]), kb, r);
        st(&o.v[i], r);
      }
      *reinterpret_cast<BnPack<T, V>*>(po + u * V) = o;
    }
    for (int64_t e = nv * V + (int64_t)blockIdx.x * 256 + threadIdx.x; e < run; e += stride) {
      float r = fmaf(ld(p0 + e), ka, kc);
      if (TWO) r = fmaf(ld(p1 + e), kb, r);
      st(po + e, r);
    }
  } else {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < run; e += stride) {
      float r = fmaf(ld(p0 + e), ka, kc);
      if (TWO) r = fmaf(ld(p1 + e), kb, r);
      st(po + e, r);
    }
  }
}

// coefficient tables from the per-channel parameters
__global__ void bn_coef_fwd_kernel(const float* mean, const float* invstd, const float* gamma, const float* beta, float* coef, int c) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  const float a = (gamma ? gamma[ch] : 1.f) * invstd[ch];
  coef[4 * ch] = a; coef[4 * ch + 1] = 0.f; coef[4 * ch + 2] = (beta ? beta[ch] : 0.f) - mean[ch] * a; coef[4 * ch + 3] = 0.f;
}
__global__ void bn_coef_bwd_kernel(const float* mean, const float* invstd, const float* gamma, const float* sum_dy,
                                   const float* sum_dy_xhat, float inv_count, float* coef, int c) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  const float k1 = (gamma ? gamma[ch] : 1.f) * invstd[ch];
  const float m1 = sum_dy[ch] * inv_count, m2 = sum_dy_xhat[ch] * inv_count;
  // dx = k1 * (dy - m1 - (x - mean) * invstd * m2)
  coef[4 * ch] = k1; coef[4 * ch + 1] = -k1 * invstd[ch] * m2; coef[4 * ch + 2] = k1 * (mean[ch] * invstd[ch] * m2 - m1); coef[4 * ch + 3] = 0.f;
}
__global__ void bn_finalize_kernel(const float* s, const float* sq, double inv_count, float eps, float* mean, float* invstd, int c) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  const double m = (double)s[ch] * inv_count;
  double var = (double)sq[ch] * inv_count - m * m;
  if (var < 0.0) var = 0.0;
  mean[ch] = (float)m;
  invstd[ch] = (float)(1.0 / sqrt(var + (double)eps));
}

h3d_status bn_check(void* handle, const h3d_tensor* x, const char* what) {
  H3D_TRY(check_tensor_packed(handle, x, what));
  if (x->c > 65535 || x->n > 65535) return fail(handle, H3D_EINVAL, "%s: more than 65535 channels or samples", what);
  return H3D_OK;
}

BnArgs bn_args(const h3d_tensor* x, const h3d_tensor* y) {
  BnArgs a;
  a.x = make_geo(x);
  a.y = y ? make_geo(y) : a.x;
  a.run = (int64_t)x->d * x->h * x->w;
  a.segs = (int)std::max<int64_t>(1, cdiv(a.run, BN_SEG));
  return a;
}

size_t bn_ws(const h3d_tensor* x) {
  const int64_t run = (int64_t)x->d * x->h * x->w;
  const int64_t segs = std::max<int64_t>(1, cdiv(run, BN_SEG));
  // partial sums [c][n * segs][2] and, behind them, the coefficient table [c][4]
  return (size_t)(((int64_t)x->c * x->n * segs * 2 + (int64_t)x->c * 4) * sizeof(float) + 255) & ~(size_t)255;
}

template <typename T, int MODE>
h3d_status bn_sums(void* handle, const h3d_tensor* x, const h3d_tensor* dy, const float* mean, const float* invstd, float* o0,
                   float* o1, void* ws, size_t ws_bytes, hipStream_t s) {
  if (x->c == 0) return H3D_OK;
  if (!o0 || !o1) return fail(handle, H3D_EINVAL, "bn: NULL output");
  if (!ws || ws_bytes < bn_ws(x)) return fail(handle, H3D_EWORKSPACE, "bn: workspace too small");
  const BnArgs a = bn_args(x, dy);
  if ((int64_t)x->n * a.run == 0) {
    hipLaunchKernelGGL(bn_reduce_kernel, dim3((unsigned)cdiv(x->c, 64)), dim3(64), 0, s, (const float*)ws, o0, o1, x->c, 0);
    return launch_status(handle, "bn_sums");
  }
  hipLaunchKernelGGL((bn_partial_kernel<T, MODE>), dim3((unsigned)a.segs, (unsigned)x->c, (unsigned)x->n), dim3(256), 0, s,
                     (const T*)x->data, dy ? (const T*)dy->data : nullptr, mean, invstd, (float*)ws, a);
  hipLaunchKernelGGL(bn_reduce_kernel, dim3((unsigned)cdiv(x->c, 64)), dim3(64), 0, s, (const float*)ws, o0, o1, x->c, x->n * a.segs);
  return launch_status(handle, "bn_sums");
}

template <typename T, bool TWO>
h3d_status bn_apply(void* handle, const h3d_tensor* in0, const h3d_tensor* in1, h3d_tensor* out, const float* coef, hipStream_t s) {
  const int64_t run = (int64_t)in0->d * in0->h * in0->w;
  if ((int64_t)in0->n * in0->c * run == 0) return H3D_OK;
  const Geo g0 = make_geo(in0), g1 = in1 ? make_geo(in1) : g0, go = make_geo(out);
  const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>(cdiv(run, 256 * 8 * 4), 1024));
  hipLaunchKernelGGL((bn_apply_kernel<T, TWO>), dim3(gx, (unsigned)in0->c, (unsigned)in0->n), dim3(256), 0, s, (const T*)in0->data,
                     in1 ? (const T*)in1->data : nullptr, (T*)out->data, coef, g0, g1, go, run);
  return launch_status(handle, "bn_apply");
}

float* bn_coef_ptr(void* ws, const h3d_tensor* x) {
  const int64_t run = (int64_t)x->d * x->h * x->w;
  const int64_t segs = std::max<int64_t>(1, cdiv(run, BN_SEG));
  return (float*)ws + (int64_t)x->c * x->n * segs * 2;
}

}  // namespace
}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_bn_workspace_bytes(void* handle, const h3d_tensor* x) {
  if (!handle || !x) return 0;
  return bn_ws(x);
}

extern "C" h3d_status h3d_bn_stats(void* handle, const h3d_tensor* x, float* sum, float* sqsum, void* ws, size_t ws_bytes,
                                   void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(bn_check(handle, x, "bn_stats: x"));
  return x->dtype == H3D_F32 ? bn_sums<float, 0>(handle, x, nullptr, nullptr, nullptr, sum, sqsum, ws, ws_bytes, (hipStream_t)stream)
                             : bn_sums<bf16_t, 0>(handle, x, nullptr, nullptr, nullptr, sum, sqsum, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" h3d_status h3d_bn_finalize(void* handle, const float* sum, const float* sqsum, int channels, int64_t count, float eps,
                                      float* mean, float* invstd, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (channels < 0 || count <= 0 || eps < 0.f) return fail(handle, H3D_EINVAL, "bn_finalize: bad channels, count or eps");
  if (channels == 0) return H3D_OK;
  if (!sum || !sqsum || !mean || !invstd) return fail(handle, H3D_EINVAL, "bn_finalize: NULL pointer");
  hipLaunchKernelGGL(bn_finalize_kernel, dim3((unsigned)cdiv(channels, 64)), dim3(64), 0, (hipStream_t)stream, sum, sqsum,
                     1.0 / (double)count, eps, mean, invstd, channels);
  return launch_status(handle, "bn_finalize");
}

extern "C" h3d_status h3d_bn_fwd(void* handle, const h3d_tensor* x, const float* mean, const float* invstd, const float* gamma,
                                 const float* beta, h3d_tensor* y, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(bn_check(handle, x, "bn_fwd: x"));
  H3D_TRY(bn_check(handle, y, "bn_fwd: y"));
  if (!same_shard(x, y) || x->c != y->c) return fail(handle, H3D_EINVAL, "bn_fwd: x and y must agree in shape, shard and dtype");
  if (x->c == 0) return H3D_OK;
  if (!mean || !invstd) return fail(handle, H3D_EINVAL, "bn_fwd: NULL statistics");
  if (!ws || ws_bytes < bn_ws(x)) return fail(handle, H3D_EWORKSPACE, "bn_fwd: workspace too small");
  float* coef = bn_coef_ptr(ws, x);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(bn_coef_fwd_kernel, dim3((unsigned)cdiv(x->c, 64)), dim3(64), 0, s, mean, invstd, gamma, beta, coef, x->c);
  return x->dtype == H3D_F32 ? bn_apply<float, false>(handle, x, nullptr, y, coef, s) : bn_apply<bf16_t, false>(handle, x, nullptr, y, coef, s);
}

extern "C" h3d_status h3d_bn_bwd_stats(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const float* mean,
                                       const float* invstd, float* sum_dy, float* sum_dy_xhat, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(bn_check(handle, x, "bn_bwd_stats: x"));
  H3D_TRY(bn_check(handle, dy, "bn_bwd_stats: dy"));
  if (!same_shard(x, dy) || x->c != dy->c) return fail(handle, H3D_EINVAL, "bn_bwd_stats: x and dy must agree in shape, shard and dtype");
  if (x->c > 0 && (!mean || !invstd)) return fail(handle, H3D_EINVAL, "bn_bwd_stats: NULL statistics");
  return x->dtype == H3D_F32 ? bn_sums<float, 1>(handle, x, dy, mean, invstd, sum_dy, sum_dy_xhat, ws, ws_bytes, (hipStream_t)stream)
                             : bn_sums<bf16_t, 1>(handle, x, dy, mean, invstd, sum_dy, sum_dy_xhat, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" h3d_status h3d_bn_bwd(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const float* mean, const float* invstd,
                                 const float* gamma, const float* sum_dy, const float* sum_dy_xhat, int64_t count, h3d_tensor* dx,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(bn_check(handle, x, "bn_bwd: x"));
  H3D_TRY(bn_check(handle, dy, "bn_bwd: dy"));
  H3D_TRY(bn_check(handle, dx, "bn_bwd: dx"));
  if (!same_shard(x, dy) || !same_shard(x, dx) || x->c != dy->c || x->c != dx->c)
    return fail(handle, H3D_EINVAL, "bn_bwd: x, dy and dx must agree in shape, shard and dtype");
  if (count <= 0) return fail(handle, H3D_EINVAL, "bn_bwd: count must be positive");
  if (x->c == 0) return H3D_OK;
  if (!mean || !invstd || !sum_dy || !sum_dy_xhat) return fail(handle, H3D_EINVAL, "bn_bwd: NULL pointer");
  if (!ws || ws_bytes < bn_ws(x)) return fail(handle, H3D_EWORKSPACE, "bn_bwd: workspace too small");
  float* coef = bn_coef_ptr(ws, x);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(bn_coef_bwd_kernel, dim3((unsigned)cdiv(x->c, 64)), dim3(64), 0, s, mean, invstd, gamma, sum_dy, sum_dy_xhat,
                     (float)(1.0 / (double)count), coef, x->c);
  return x->dtype == H3D_F32 ? bn_apply<float, true>(handle, dy, x, dx, coef, s) : bn_apply<bf16_t, true>(handle, dy, x, dx, coef, s);
}
