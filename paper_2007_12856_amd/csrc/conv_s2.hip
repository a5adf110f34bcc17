// Stride-2 3x3x3 convolution (Table I: the fourth convolution of the CosmoFlow network), forward,
// backward-data and backward-filter, on a depth slab.
//
// y[p] = sum_k w[k] x~[2p+k-1] is rewritten as a stride-1 convolution over the eight parity
// sub-lattices of x.  With x'[(par,ci)][q] = x[ci][2q+par] (par = (pd,ph,pw) in {0,1}^3), per axis
//     k = 0 reads parity 1 at q = p-1,   k = 1 reads parity 0 at q = p,   k = 2 reads parity 1 at q = p,
// so y = W' (*) x' with a stride-1 3x3x3 filter W' over 8 Cin channels whose taps at shift +1 (and the
// parity/shift pairs that no k maps to) are zero.  The stride-1 kernels of this library (matrix cores for
// bf16) then run all three passes; the zero padding of the stride-1 call at q = -1 is exactly the zero
// padding of x at index -1.  The price is that 27 of the 216 (parity, tap) products per input channel are
// non-zero; the gain is the matrix-core kernels instead of a scalar gather for a layer that is a small
// part of the network's work.
//
// Small element-wise kernels here: the parity split of x, its inverse for dx, the masked copy of dy into
// a slab with both halo planes, the filter expansion and the extraction of dw from dW'.
#include <algorithm>

#include "common.h"

namespace h3d {

static constexpr int S2_THREADS = 256;

// x' [n][8 cin][1 + d2 + 1][h2][w2]; planes -1 and d2 are halos.  Only the parity-1 half of plane -1 can
// carry data (x plane -1); everything that has no source voxel is zero.
template <typename T>
__global__ void __launch_bounds__(S2_THREADS) s2_split_kernel(const T* __restrict__ x, Geo xg, T* __restrict__ xs, int d2,
                                                              int h2, int w2, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * S2_THREADS + threadIdx.x;
  if (i >= total) return;
  const int v = (int)(i % w2); int64_t r = i / w2;
  const int hh = (int)(r % h2); r /= h2;
  const int qs = (int)(r % (d2 + 2)); r /= (d2 + 2);
  const int cp = (int)(r % (8 * xg.c));
  const int n = (int)(r / (8 * xg.c));
  const int par = cp / xg.c, ci = cp % xg.c;
  const int p = 2 * (qs - 1) + (par >> 2), h = 2 * hh + ((par >> 1) & 1), w = 2 * v + (par & 1);
  T val = (T)0;
  const int64_t gp = xg.doff + p;
  if (p >= -xg.hlo && p < xg.d && gp >= 0 && gp < xg.dglob && h < xg.h && w < xg.w)
    val = x[n * xg.nstride + ci * xg.cstride + (int64_t)(p + xg.hlo) * xg.plane + (int64_t)h * xg.w + w];
  xs[i] = val;
}

// dx[n][ci][q][h][w] = dx'[n][(par,ci)][q/2][h/2][w/2]
template <typename T>
__global__ void __launch_bounds__(S2_THREADS) s2_merge_kernel(const T* __restrict__ ds, T* __restrict__ dx, Geo xg, int d2,
                                                              int h2, int w2, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * S2_THREADS + threadIdx.x;
  if (i >= total) return;
  const int w = (int)(i % xg.w); int64_t r = i / xg.w;
  const int h = (int)(r % xg.h); r /= xg.h;
  const int q = (int)(r % xg.d); r /= xg.d;
  const int ci = (int)(r % xg.c);
  const int n = (int)(r / xg.c);
  const int par = ((q & 1) << 2) | ((h & 1) << 1) | (w & 1);
  const int64_t src = ((((int64_t)n * 8 * xg.c + par * xg.c + ci) * d2 + (q >> 1)) * h2 + (h >> 1)) * w2 + (w >> 1);
  dx[n * xg.nstride + ci * xg.cstride + (int64_t)(q + xg.hlo) * xg.plane + (int64_t)h * xg.w + w] = ds[src];
}

// g [n][c][1 + d2 + 1][h2][w2] = dy * (y > 0 ? 1 : slope) on planes 0..d2 (plane d2 only if it is inside
// the volume: it is dy's upper halo plane), zero on plane -1 and outside the volume.
template <typename T, bool MASKED>
__global__ void __launch_bounds__(S2_THREADS) s2_grad_kernel(const T* __restrict__ dy, Geo yg, const T* __restrict__ y, Geo ysg,
                                                             T* __restrict__ g, float slope, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * S2_THREADS + threadIdx.x;
  if (i >= total) return;
  const int64_t plane = yg.plane;
  const int64_t hw = i % plane; int64_t r = i / plane;
  const int qs = (int)(r % (yg.d + 2)); r /= (yg.d + 2);
  const int c = (int)(r % yg.c);
  const int n = (int)(r / yg.c);
  const int p = qs - 1;
  T val = (T)0;
  if (p >= 0 && yg.doff + p < yg.dglob) {
    val = dy[n * yg.nstride + c * yg.cstride + (int64_t)(p + yg.hlo) * plane + hw];
    if (MASKED) {
      const float m = ld(y + n * ysg.nstride + c * ysg.cstride + (int64_t)(p + ysg.hlo) * plane + hw);
      if (!(m > 0.f)) { T t; st(&t, ld(&val) * slope); val = t; }
    }
  }
  g[i] = val;
}

// per axis: which k does (parity, shift s in {-1,0,1}) stand for; -1 = none
__host__ __device__ __forceinline__ int s2_tap(int par, int s) { return par == 0 ? (s == 0 ? 1 : -1) : (s == -1 ? 0 : (s == 0 ? 2 : -1)); }

// W' [cout][8 cin][27] from w [cout][cin][27]
template <typename T>
__global__ void __launch_bounds__(S2_THREADS) s2_expand_w_kernel(const T* __restrict__ w, T* __restrict__ we, int cin, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * S2_THREADS + threadIdx.x;
  if (i >= total) return;
  const int t = (int)(i % 27); int64_t r = i / 27;
  const int cp = (int)(r % (8 * cin));
  const int64_t co = r / (8 * cin);
  const int par = cp / cin, ci = cp % cin;
  const int kd = s2_tap(par >> 2, t / 9 - 1), kh = s2_tap((par >> 1) & 1, (t / 3) % 3 - 1), kw = s2_tap(par & 1, t % 3 - 1);
  T val = (T)0;
  if (kd >= 0 && kh >= 0 && kw >= 0) val = w[(co * cin + ci) * 27 + kd * 9 + kh * 3 + kw];
  we[i] = val;
}

// dw [cout][cin][27] from dW' [cout][8 cin][27]: tap k sits at parity (k != 1), shift (k == 0 ? -1 : 0)
__global__ void __launch_bounds__(S2_THREADS) s2_extract_dw_kernel(const float* __restrict__ dwe, float* __restrict__ dw, int cin,
                                                                   int64_t total) {
  int64_t i = (int64_t)blockIdx.x * S2_THREADS + threadIdx.x;
  if (i >= total) return;
  const int t = (int)(i % 27); int64_t r = i / 27;
  const int ci = (int)(r % cin);
  const int64_t co = r / cin;
  const int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
  const int par = ((kd != 1) << 2) | ((kh != 1) << 1) | (kw != 1);
  const int te = (kd == 0 ? 0 : 1) * 9 + (kh == 0 ? 0 : 1) * 3 + (kw == 0 ? 0 : 1);
  dw[i] = dwe[(co * 8 * cin + par * cin + ci) * 27 + te];
}

static inline size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

// the descriptors of the stride-1 problem
struct S2Plan {
  h3d_tensor xs;   // x' (8 cin channels, halo 1/1)
  h3d_tensor gs;   // g  (cout channels, halo 1/1)
  h3d_tensor yv;   // interior of y: y itself when it stores no halo planes, else a plane-run view (cout channels, no halo)
  h3d_tensor dxs;  // dx' (8 cin channels, no halo)
  size_t xs_bytes, gs_bytes, dxs_bytes, we_bytes, dwe_bytes;
};

static S2Plan s2_plan(const h3d_tensor* x, const h3d_tensor* y) {
  S2Plan p;
  const size_t es = elt_size(x->dtype);
  h3d_tensor t;
  memset(&t, 0, sizeof(t));
  t.dtype = x->dtype; t.n = x->n; t.d = y->d; t.h = y->h; t.w = y->w;
  t.d_offset = y->d_offset; t.d_global = y->d_global;
  p.xs = t; p.xs.c = 8 * x->c; p.xs.halo_lo = p.xs.halo_hi = 1;
  p.gs = t; p.gs.c = y->c; p.gs.halo_lo = p.gs.halo_hi = 1;
  p.dxs = t; p.dxs.c = 8 * x->c;
  p.yv = t; p.yv.c = y->c;
  const int64_t yplane = (int64_t)y->h * y->w, yds = y->halo_lo + y->d + y->halo_hi;
  if (y->halo_lo || y->halo_hi) {   // without halo planes y itself is the packed interior: the inner call may then take
    p.yv.c_stride = yplane * yds;   // the channel-split kernel, which plane-run views never do (8 x cin input channels on a
    p.yv.n_stride = p.yv.c_stride * y->c;   // small volume is exactly its case)
  }
  p.yv.data = y->data ? (char*)y->data + (size_t)y->halo_lo * yplane * es : nullptr;
  const size_t vol = (size_t)y->h * y->w;
  p.xs_bytes = up256((size_t)x->n * 8 * x->c * (y->d + 2) * vol * es);
  p.gs_bytes = up256((size_t)x->n * y->c * (y->d + 2) * vol * es);
  p.dxs_bytes = up256((size_t)x->n * 8 * x->c * y->d * vol * es);
  p.we_bytes = up256((size_t)y->c * 8 * x->c * 27 * es);
  p.dwe_bytes = up256((size_t)y->c * 8 * x->c * 27 * sizeof(float));
  return p;
}

static h3d_status s2_check(void* handle, const h3d_tensor* x, const h3d_tensor* y, const char* what) {
  H3D_TRY(check_tensor_packed(handle, x, "x"));
  H3D_TRY(check_tensor_packed(handle, y, "y"));
  if (x->dtype != y->dtype || x->n != y->n) return fail(handle, H3D_EINVAL, "%s: dtype or sample count differ", what);
  if ((x->d | x->d_offset | x->d_global) & 1)
    return fail(handle, H3D_EUNSUPPORTED, "%s: d, d_offset and d_global of the input must be even (no window may straddle a shard face)", what);
  if (y->d != x->d / 2 || y->h != (x->h + 1) / 2 || y->w != (x->w + 1) / 2 || y->d_offset != x->d_offset / 2 || y->d_global != x->d_global / 2)
    return fail(handle, H3D_EINVAL, "%s: the output shard must have d/2, ceil(h/2), ceil(w/2), d_offset/2, d_global/2 of the input", what);
  if ((int64_t)x->c * 8 > INT32_MAX / 64) return fail(handle, H3D_EINVAL, "%s: too many channels", what);
  return H3D_OK;
}

static inline unsigned s2_grid(int64_t total) { return (unsigned)cdiv(total, S2_THREADS); }

template <typename T>
static void launch_split(const h3d_tensor* x, const S2Plan& p, void* xs, hipStream_t s) {
  const int64_t total = (int64_t)x->n * 8 * x->c * (p.xs.d + 2) * p.xs.h * p.xs.w;
  if (total) hipLaunchKernelGGL((s2_split_kernel<T>), dim3(s2_grid(total)), dim3(S2_THREADS), 0, s, (const T*)x->data, make_geo(x), (T*)xs, p.xs.d, p.xs.h, p.xs.w, total);
}

template <typename T>
static void launch_expand(const void* w, void* we, int cin, int cout, hipStream_t s) {
  const int64_t total = (int64_t)cout * 8 * cin * 27;
  if (total) hipLaunchKernelGGL((s2_expand_w_kernel<T>), dim3(s2_grid(total)), dim3(S2_THREADS), 0, s, (const T*)w, (T*)we, cin, total);
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_conv3d_s2_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* y) {
  if (!handle || !x || !y || x->c < 0 || y->c < 0) return 0;
  h3d_tensor xc = *x, yc = *y;
  xc.data = yc.data = nullptr;
  const S2Plan p = s2_plan(&xc, &yc);
  switch (op) {
    case H3D_OP_FWD:
      return p.xs_bytes + p.we_bytes + h3d_conv3d_workspace_bytes(handle, H3D_OP_FWD, &p.xs, &p.yv);
    case H3D_OP_BWD_DATA:
      return p.gs_bytes + p.dxs_bytes + p.we_bytes + h3d_conv3d_workspace_bytes(handle, H3D_OP_BWD_DATA, &p.gs, &p.dxs);
    case H3D_OP_BWD_FILTER:
      return p.xs_bytes + p.dwe_bytes + h3d_conv3d_workspace_bytes(handle, H3D_OP_BWD_FILTER, &p.xs, &p.yv);
    default:
      return 0;
  }
}

extern "C" h3d_status h3d_conv3d_s2_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y, int act,
                                        float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!x || !y) return fail(handle, H3D_EINVAL, "conv3d_s2_fwd: NULL descriptor");
  H3D_TRY(s2_check(handle, x, y, "conv3d_s2_fwd"));
  if (!w && x->c * y->c > 0) return fail(handle, H3D_EINVAL, "conv3d_s2_fwd: NULL weights");
  if (y->d > 0 && x->d_offset > 0 && x->halo_lo < 1) return fail(handle, H3D_EHALO, "conv3d_s2_fwd: x must store its lower halo plane");
  if (!ws || ws_bytes < h3d_conv3d_s2_workspace_bytes(handle, H3D_OP_FWD, x, y)) return fail(handle, H3D_EWORKSPACE, "conv3d_s2_fwd: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_s2_fwd: workspace must be 256-byte aligned");
  S2Plan p = s2_plan(x, y);
  char* base = (char*)ws;
  p.xs.data = base;
  void* we = base + p.xs_bytes;
  void* inner = base + p.xs_bytes + p.we_bytes;
  hipStream_t s = (hipStream_t)stream;
  if (x->dtype == H3D_F32) { launch_split<float>(x, p, p.xs.data, s); launch_expand<float>(w, we, x->c, y->c, s); }
  else { launch_split<bf16_t>(x, p, p.xs.data, s); launch_expand<bf16_t>(w, we, x->c, y->c, s); }
  H3D_TRY(launch_status(handle, "conv3d_s2_fwd (split)"));
  return h3d_conv3d_fwd(handle, &p.xs, we, bias, &p.yv, act, alpha, inner, ws_bytes - p.xs_bytes - p.we_bytes, stream);
}

extern "C" h3d_status h3d_conv3d_s2_bwd_data(void* handle, const h3d_tensor* dy, const h3d_tensor* y, const void* w, h3d_tensor* dx,
                                             int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!dy || !dx) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_data: NULL descriptor");
  H3D_TRY(s2_check(handle, dx, dy, "conv3d_s2_bwd_data"));
  if (!w && dx->c * dy->c > 0) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_data: NULL weights");
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  if (act == H3D_ACT_NONE) y = nullptr;
  const bool upper = dy->d > 0 && dy->d_offset + dy->d < dy->d_global;
  if (upper && dy->halo_hi < 1) return fail(handle, H3D_EHALO, "conv3d_s2_bwd_data: dy must store its upper halo plane");
  if (y) {
    H3D_TRY(check_tensor_packed(handle, y, "y"));
    if (!same_shard(y, dy) || y->c != dy->c) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_data: y and dy shapes differ");
    if (upper && y->halo_hi < 1) return fail(handle, H3D_EHALO, "conv3d_s2_bwd_data: y must store its upper halo plane");
  }
  if (!ws || ws_bytes < h3d_conv3d_s2_workspace_bytes(handle, H3D_OP_BWD_DATA, dx, dy)) return fail(handle, H3D_EWORKSPACE, "conv3d_s2_bwd_data: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_data: workspace must be 256-byte aligned");
  S2Plan p = s2_plan(dx, dy);
  char* base = (char*)ws;
  p.gs.data = base;
  p.dxs.data = base + p.gs_bytes;
  void* we = base + p.gs_bytes + p.dxs_bytes;
  void* inner = base + p.gs_bytes + p.dxs_bytes + p.we_bytes;
  hipStream_t s = (hipStream_t)stream;
  const float slope = act_slope(act, alpha);
  const int64_t gtotal = (int64_t)dy->n * dy->c * (dy->d + 2) * dy->h * dy->w;
  const int64_t xtotal = (int64_t)dx->n * dx->c * dx->d * dx->h * dx->w;
  const Geo yg = make_geo(dy), ysg = y ? make_geo(y) : yg;
#define S2_GRAD(T, M) hipLaunchKernelGGL((s2_grad_kernel<T, M>), dim3(s2_grid(gtotal)), dim3(S2_THREADS), 0, s, (const T*)dy->data, yg, \
                                         (const T*)(y ? y->data : nullptr), ysg, (T*)p.gs.data, slope, gtotal)
  if (gtotal) {
    if (dy->dtype == H3D_F32) { if (y) S2_GRAD(float, true); else S2_GRAD(float, false); }
    else { if (y) S2_GRAD(bf16_t, true); else S2_GRAD(bf16_t, false); }
  }
#undef S2_GRAD
  if (dy->dtype == H3D_F32) launch_expand<float>(w, we, dx->c, dy->c, s); else launch_expand<bf16_t>(w, we, dx->c, dy->c, s);
  H3D_TRY(launch_status(handle, "conv3d_s2_bwd_data (grad copy)"));
  H3D_TRY(h3d_conv3d_bwd_data(handle, &p.gs, nullptr, we, &p.dxs, H3D_ACT_NONE, 0.f, inner, ws_bytes - p.gs_bytes - p.dxs_bytes - p.we_bytes, stream));
  if (xtotal) {
    if (dx->dtype == H3D_F32)
      hipLaunchKernelGGL((s2_merge_kernel<float>), dim3(s2_grid(xtotal)), dim3(S2_THREADS), 0, s, (const float*)p.dxs.data, (float*)dx->data, make_geo(dx), dy->d, dy->h, dy->w, xtotal);
    else
      hipLaunchKernelGGL((s2_merge_kernel<bf16_t>), dim3(s2_grid(xtotal)), dim3(S2_THREADS), 0, s, (const bf16_t*)p.dxs.data, (bf16_t*)dx->data, make_geo(dx), dy->d, dy->h, dy->w, xtotal);
  }
  return launch_status(handle, "conv3d_s2_bwd_data (merge)");
}

extern "C" h3d_status h3d_conv3d_s2_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dy, const h3d_tensor* y, float* dw,
                                               float* db, int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!x || !dy) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_filter: NULL descriptor");
  H3D_TRY(s2_check(handle, x, dy, "conv3d_s2_bwd_filter"));
  if (!dw && x->c * dy->c > 0) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_filter: NULL dw");
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  if (act == H3D_ACT_NONE) y = nullptr;
  if (dy->d > 0 && x->d_offset > 0 && x->halo_lo < 1) return fail(handle, H3D_EHALO, "conv3d_s2_bwd_filter: x must store its lower halo plane");
  if (y) {
    H3D_TRY(check_tensor_packed(handle, y, "y"));
    if (!same_shard(y, dy) || y->c != dy->c) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_filter: y and dy shapes differ");
  }
  if (!ws || ws_bytes < h3d_conv3d_s2_workspace_bytes(handle, H3D_OP_BWD_FILTER, x, dy)) return fail(handle, H3D_EWORKSPACE, "conv3d_s2_bwd_filter: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_s2_bwd_filter: workspace must be 256-byte aligned");
  S2Plan p = s2_plan(x, dy);
  char* base = (char*)ws;
  p.xs.data = base;
  float* dwe = (float*)(base + p.xs_bytes);
  void* inner = base + p.xs_bytes + p.dwe_bytes;
  hipStream_t s = (hipStream_t)stream;
  if (x->dtype == H3D_F32) launch_split<float>(x, p, p.xs.data, s); else launch_split<bf16_t>(x, p, p.xs.data, s);
  H3D_TRY(launch_status(handle, "conv3d_s2_bwd_filter (split)"));
  h3d_tensor yv = p.yv;   // interior plane run of y, same strides as dy's when both carry the same halos
  h3d_tensor* yvp = nullptr;
  if (y) {
    S2Plan py = s2_plan(x, y);
    yv = py.yv;
    yvp = &yv;
  }
  H3D_TRY(h3d_conv3d_bwd_filter(handle, &p.xs, &p.yv, yvp, dwe, db, act, alpha, inner, ws_bytes - p.xs_bytes - p.dwe_bytes, stream));
  const int64_t total = (int64_t)dy->c * x->c * 27;
  if (total) hipLaunchKernelGGL(s2_extract_dw_kernel, dim3(s2_grid(total)), dim3(S2_THREADS), 0, s, (const float*)dwe, dw, x->c, total);
  return launch_status(handle, "conv3d_s2_bwd_filter (extract)");
}
