// Per-voxel softmax cross-entropy of a segmentation output on a depth slab, forward and gradient in one streaming
// pass (Sec. III-A: the cross-entropy loss is one of the components that needed a version for large 3-D data; the
// ground-truth labels are partitioned like the activations).  HBM-bound: per voxel C logits and one label byte in,
// C gradient values out.  A thread takes 8 consecutive voxels of a row (one 16-byte load per class in bf16) when
// the rows allow it, else one voxel.  The loss is summed per thread, per wavefront (butterfly), per block (in
// wavefront order), and a second one-block kernel adds the block partials in block order: same bits every run.
#include "common.h"

namespace h3d {

constexpr int XE_THREADS = 256;
constexpr int XE_MAXC_VEC = 8;     // classes held in registers by the 8-voxel path

struct XentArgs {
  Geo z, g;
  int c;
  int64_t units;     // work items: n * d * h * (w / V)
  float inv_count;
};

__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float s = red[0];
  for (int i = 1; i < XE_THREADS / 64; ++i) s += red[i];
  return s;
}

// V = 8, bf16, at most XE_MAXC_VEC classes
template <int C>
__global__ void __launch_bounds__(XE_THREADS) xent_vec8_kernel(const bf16_t* __restrict__ z, const uint8_t* __restrict__ lab,
                                                               bf16_t* __restrict__ g, float* __restrict__ part, XentArgs a) {
  __shared__ float red[XE_THREADS / 64];
  const int wu = a.z.w / 8;
  float loss = 0.f;
  for (int64_t u = (int64_t)blockIdx.x * XE_THREADS + threadIdx.x; u < a.units; u += (int64_t)gridDim.x * XE_THREADS) {
    int64_t r = u;
    const int wq = (int)(r % wu); r /= wu;
    const int h = (int)(r % a.z.h); r /= a.z.h;
    const int p = (int)(r % a.z.d);
    const int n = (int)(r / a.z.d);
    const int64_t zo = n * a.z.nstride + (int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)h * a.z.w + 8 * wq;
    const int64_t go = n * a.g.nstride + (int64_t)(p + a.g.hlo) * a.g.plane + (int64_t)h * a.g.w + 8 * wq;
    const uint2 lb = *reinterpret_cast<const uint2*>(lab + (((int64_t)n * a.z.d + p) * a.z.h + h) * a.z.w + 8 * wq);
    float v[C][8];
#pragma unroll
    for (int k = 0; k < C; ++k) {
      const uint4 q = *reinterpret_cast<const uint4*>(z + zo + k * a.z.cstride);
      const uint32_t d4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[k][2 * e] = __uint_as_float(d4[e] << 16);
        v[k][2 * e + 1] = __uint_as_float(d4[e] & 0xffff0000u);
      }
    }
    uint32_t out[C][4];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int label = (int)(((e < 4 ? lb.x : lb.y) >> (8 * (e & 3))) & 0xffu);
      float m = v[0][e];
#pragma unroll
      for (int k = 1; k < C; ++k) m = fmaxf(m, v[k][e]);
      float se = 0.f, ex[C], picked = 0.f;
#pragma unroll
      for (int k = 0; k < C; ++k) {
        ex[k] = expf(v[k][e] - m);
        se += ex[k];
        if (k == label) picked = v[k][e];
      }
      const bool valid = label < C;
      if (valid) loss += logf(se) + m - picked;
      const float scale = valid ? a.inv_count / se : 0.f;
#pragma unroll
      for (int k = 0; k < C; ++k) {
        const float gv = ex[k] * scale - ((valid && k == label) ? a.inv_count : 0.f);
        const uint32_t b = f32_to_bf16(gv);
        if (e & 1) out[k][e >> 1] |= b << 16; else out[k][e >> 1] = b;
      }
    }
#pragma unroll
    for (int k = 0; k < C; ++k)
      *reinterpret_cast<uint4*>(g + go + k * a.g.cstride) = uint4{out[k][0], out[k][1], out[k][2], out[k][3]};
  }
  const float s = block_sum(loss, red);
  if (threadIdx.x == 0) part[blockIdx.x] = s;
}

// one voxel per thread, any class count, either dtype: three passes over the classes (maximum, sum, gradient)
template <typename T>
__global__ void __launch_bounds__(XE_THREADS) xent_scalar_kernel(const T* __restrict__ z, const uint8_t* __restrict__ lab,
                                                                 T* __restrict__ g, float* __restrict__ part, XentArgs a) {
  __shared__ float red[XE_THREADS / 64];
  float loss = 0.f;
  for (int64_t u = (int64_t)blockIdx.x * XE_THREADS + threadIdx.x; u < a.units; u += (int64_t)gridDim.x * XE_THREADS) {
    int64_t r = u;
    const int w = (int)(r % a.z.w); r /= a.z.w;
    const int h = (int)(r % a.z.h); r /= a.z.h;
    const int p = (int)(r % a.z.d);
    const int n = (int)(r / a.z.d);
    const T* zp = z + n * a.z.nstride + (int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)h * a.z.w + w;
    T* gp = g + n * a.g.nstride + (int64_t)(p + a.g.hlo) * a.g.plane + (int64_t)h * a.g.w + w;
    const int label = lab[u];
    float m = ld(zp);
    for (int k = 1; k < a.c; ++k) m = fmaxf(m, ld(zp + k * a.z.cstride));
    float se = 0.f, picked = 0.f;
    for (int k = 0; k < a.c; ++k) {
      const float vk = ld(zp + k * a.z.cstride);
      se += expf(vk - m);
      if (k == label) picked = vk;
    }
    const bool valid = label < a.c;
    if (valid) loss += logf(se) + m - picked;
    const float scale = valid ? a.inv_count / se : 0.f;
    for (int k = 0; k < a.c; ++k) {
      const float vk = ld(zp + k * a.z.cstride);
      st(gp + k * a.g.cstride, expf(vk - m) * scale - ((valid && k == label) ? a.inv_count : 0.f));
    }
  }
  const float s = block_sum(loss, red);
  if (threadIdx.x == 0) part[blockIdx.x] = s;
}

// block partials -> loss: thread t adds partials t, t + 256, ... in that order, then the fixed block tree
__global__ void __launch_bounds__(XE_THREADS) xent_reduce_kernel(const float* __restrict__ part, int nparts, float inv_count,
                                                                 float* __restrict__ loss) {
  __shared__ float red[XE_THREADS / 64];
  float s = 0.f;
  for (int i = threadIdx.x; i < nparts; i += XE_THREADS) s += part[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) loss[0] = s * inv_count;
}

static int xent_blocks(void* handle, int64_t units) {
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  return (int)std::max<int64_t>(1, std::min<int64_t>((int64_t)num_cu * 8, cdiv(units, XE_THREADS)));
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_softmax_xent_workspace_bytes(void* handle, const h3d_tensor* logits) {
  if (!handle || !logits) return 0;
  return (size_t)static_cast<Handle*>(handle)->num_cu * 8 * sizeof(float);
}

extern "C" h3d_status h3d_softmax_xent_fwd_bwd(void* handle, const h3d_tensor* logits, const uint8_t* labels, int64_t count, float* loss,
                                               h3d_tensor* dlogits, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor_packed(handle, logits, "logits"));
  H3D_TRY(check_tensor_packed(handle, dlogits, "dlogits"));
  if (!same_shard(logits, dlogits) || logits->c != dlogits->c) return fail(handle, H3D_EINVAL, "softmax_xent: logits and dlogits must describe the same shard");
  if (logits->c < 1 || logits->c > 255) return fail(handle, H3D_EINVAL, "softmax_xent: 1..255 classes");
  if (count < 1) return fail(handle, H3D_EINVAL, "softmax_xent: count must be positive");
  if (!loss) return fail(handle, H3D_EINVAL, "softmax_xent: NULL loss");
  if (!ws || ws_bytes < h3d_softmax_xent_workspace_bytes(handle, logits)) return fail(handle, H3D_EWORKSPACE, "softmax_xent: workspace too small");
  const int64_t vox = (int64_t)logits->n * logits->d * logits->h * logits->w;
  if (vox > 0 && !labels) return fail(handle, H3D_EINVAL, "softmax_xent: NULL labels");
  XentArgs a;
  a.z = make_geo(logits); a.g = make_geo(dlogits); a.c = logits->c;
  a.inv_count = (float)(1.0 / (double)count);
  hipStream_t s = (hipStream_t)stream;
  float* part = (float*)ws;
  int blocks = 1;
  if (vox == 0) {
    blocks = 0;
  } else {
    const bool vec = logits->dtype == H3D_BF16 && logits->c <= XE_MAXC_VEC && logits->w % 8 == 0 && ((uintptr_t)logits->data % 16 == 0) &&
                     ((uintptr_t)dlogits->data % 16 == 0) && ((uintptr_t)labels % 8 == 0);
    a.units = vec ? vox / 8 : vox;
    blocks = xent_blocks(handle, a.units);
    const bf16_t* zp = (const bf16_t*)logits->data;
    bf16_t* gp = (bf16_t*)dlogits->data;
#define XE_CASE(C) case C: hipLaunchKernelGGL((xent_vec8_kernel<C>), dim3(blocks), dim3(XE_THREADS), 0, s, zp, labels, gp, part, a); break;
    if (vec) {
      switch (logits->c) {
        XE_CASE(1) XE_CASE(2) XE_CASE(3) XE_CASE(4) XE_CASE(5) XE_CASE(6) XE_CASE(7) XE_CASE(8)
      }
    } else if (logits->dtype == H3D_F32) {
      hipLaunchKernelGGL((xent_scalar_kernel<float>), dim3(blocks), dim3(XE_THREADS), 0, s, (const float*)logits->data, labels, (float*)dlogits->data, part, a);
    } else {
      hipLaunchKernelGGL((xent_scalar_kernel<bf16_t>), dim3(blocks), dim3(XE_THREADS), 0, s, zp, labels, gp, part, a);
    }
#undef XE_CASE
  }
  hipLaunchKernelGGL(xent_reduce_kernel, dim3(1), dim3(XE_THREADS), 0, s, (const float*)part, blocks, a.inv_count, loss);
  return launch_status(handle, "softmax_xent");
}
