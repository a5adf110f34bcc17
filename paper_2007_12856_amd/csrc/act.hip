// Activation backward as its own streaming pass: g = (dz [+ dz2]) * (z > 0 ? 1 : slope) on the
// shard interior.  The product g is what the halo exchange of the backward pass carries (one
// tensor instead of dz and z), and both backward convolutions then run without a mask.  The
// optional second gradient merges the two branches that meet at a U-Net skip connection.
#include "common.h"

namespace h3d {

struct ActArgs {
  Geo dz, dz2, z, g;
  int64_t total;   // n*c*d*h*(w/VEC)
  int wv;
  float slope;
};

template <typename T, int N>
struct alignas(sizeof(T) * N) AVec {
  T v[N];
};

template <typename T, int VEC, bool TWO>
__global__ void __launch_bounds__(256) act_bwd_kernel(const T* __restrict__ dz, const T* __restrict__ dz2, const T* __restrict__ z,
                                                      T* __restrict__ g, ActArgs a) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int wv = (int)(t % a.wv); t /= a.wv;
  int h = (int)(t % a.g.h); t /= a.g.h;
  int p = (int)(t % a.g.d); t /= a.g.d;
  int c = (int)(t % a.g.c);
  int n = (int)(t / a.g.c);
  auto off = [&](const Geo& q) { return n * q.nstride + c * q.cstride + (int64_t)(p + q.hlo) * q.plane + (int64_t)h * q.w + wv * VEC; };
  AVec<T, VEC> d = *reinterpret_cast<const AVec<T, VEC>*>(dz + off(a.dz));
  AVec<T, VEC> m = *reinterpret_cast<const AVec<T, VEC>*>(z + off(a.z));
  AVec<T, VEC> d2, o;
  if (TWO) d2 = *reinterpret_cast<const AVec<T, VEC>*>(dz2 + off(a.dz2));
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    float v = ld(&d.v[i]);
    if (TWO) v += ld(&d2.v[i]);
    if (!(ld(&m.v[i]) > 0.f)) v *= a.slope;
    st(&o.v[i], v);
  }
  *reinterpret_cast<AVec<T, VEC>*>(g + off(a.g)) = o;
}

template <typename T>
static h3d_status act_bwd_t(void* handle, const h3d_tensor* dz, const h3d_tensor* dz2, const h3d_tensor* z, h3d_tensor* g,
                            float slope, hipStream_t s) {
  ActArgs a;
  a.dz = make_geo(dz); a.dz2 = dz2 ? make_geo(dz2) : a.dz; a.z = make_geo(z); a.g = make_geo(g);
  a.slope = slope;
  constexpr int V = 16 / sizeof(T);
  auto aligned = [&](const h3d_tensor* t) { return !t || (uintptr_t)t->data % 16 == 0; };
  const bool vec = g->w % V == 0 && aligned(dz) && aligned(dz2) && aligned(z) && aligned(g);
  a.wv = vec ? g->w / V : g->w;
  a.total = (int64_t)g->n * g->c * g->d * g->h * a.wv;
  if (a.total == 0) return H3D_OK;
  int64_t grid = cdiv(a.total, 256);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "act_bwd: too many blocks");
  const T *pd = (const T*)dz->data, *p2 = dz2 ? (const T*)dz2->data : nullptr, *pz = (const T*)z->data;
  T* pg = (T*)g->data;
  if (vec) {
    if (dz2) hipLaunchKernelGGL((act_bwd_kernel<T, V, true>), dim3((unsigned)grid), dim3(256), 0, s, pd, p2, pz, pg, a);
    else hipLaunchKernelGGL((act_bwd_kernel<T, V, false>), dim3((unsigned)grid), dim3(256), 0, s, pd, p2, pz, pg, a);
  } else {
    if (dz2) hipLaunchKernelGGL((act_bwd_kernel<T, 1, true>), dim3((unsigned)grid), dim3(256), 0, s, pd, p2, pz, pg, a);
    else hipLaunchKernelGGL((act_bwd_kernel<T, 1, false>), dim3((unsigned)grid), dim3(256), 0, s, pd, p2, pz, pg, a);
  }
  return launch_status(handle, "act_bwd");
}

}  // namespace h3d

using namespace h3d;

extern "C" h3d_status h3d_act_bwd(void* handle, const h3d_tensor* dz, const h3d_tensor* dz2, const h3d_tensor* z, h3d_tensor* g,
                                  int act, float alpha, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor(handle, dz, "dz"));
  H3D_TRY(check_tensor(handle, z, "z"));
  H3D_TRY(check_tensor(handle, g, "g"));
  if (dz2) H3D_TRY(check_tensor(handle, dz2, "dz2"));
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "act_bwd: bad activation");
  if (!same_shard(dz, g) || !same_shard(z, g) || dz->c != g->c || z->c != g->c || (dz2 && (!same_shard(dz2, g) || dz2->c != g->c)))
    return fail(handle, H3D_EINVAL, "act_bwd: all tensors must agree in n,c,d,h,w,d_offset,d_global,dtype");
  const float slope = act_slope(act, alpha);
  return g->dtype == H3D_F32 ? act_bwd_t<float>(handle, dz, dz2, z, g, slope, (hipStream_t)stream)
                             : act_bwd_t<bf16_t>(handle, dz, dz2, z, g, slope, (hipStream_t)stream);
}
