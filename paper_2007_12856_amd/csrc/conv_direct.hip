// Direct (non-MFMA) 3x3x3 convolution kernels: the general path for any channel count and for
// fp32 storage, where the contraction is too thin or too irregular for the matrix cores
// (Cin = 1 or 3, Cout not a multiple of 16, true-fp32 arithmetic).  fp32 accumulation throughout.
//
//  * forward and backward-data share one kernel: backward-data is a forward correlation of
//    g = dz * act'(z) with the weights transposed (ci <-> co) and reversed on every axis;
//    a small pack kernel writes the weights as fp32 [cin][27][cout_pad] so that the COT output
//    channels of a (ci,tap) are contiguous and wave-uniform (scalar loads).
//  * backward-filter is two-stage and deterministic: stage 1 gives every block a fixed chunk of
//    the voxel range and reduces inside the block in a fixed tree; stage 2 adds the chunk
//    partials in chunk order.
#include <algorithm>

#include "common.h"

namespace h3d {

constexpr int COT = 16;  // output channels per thread in the direct forward kernel

// w: [cout][cin][27] (T)  ->  wk: fp32 [cin_k][27][cout_k_pad]
// fwd:      wk[ci][t][co]      = w[co][ci][t]
// bwd-data: wk[co][t][ci]      = w[co][ci][26 - t]      (cin_k = cout, cout_k = cin)
template <typename T>
__global__ void pack_w_direct_kernel(const T* __restrict__ w, float* __restrict__ wk, int cin, int cout, int transpose,
                                     int cout_k_pad) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int cin_k = transpose ? cout : cin;
  int64_t total = (int64_t)cin_k * 27 * cout_k_pad;
  if (i >= total) return;
  int ok = (int)(i % cout_k_pad);
  int t = (int)((i / cout_k_pad) % 27);
  int ik = (int)(i / ((int64_t)cout_k_pad * 27));
  int cout_k = transpose ? cin : cout;
  float v = 0.f;
  if (ok < cout_k) {
    v = transpose ? ld(&w[((int64_t)ik * cin + ok) * 27 + (26 - t)]) : ld(&w[((int64_t)ok * cin + ik) * 27 + t]);
  }
  wk[i] = v;
}

struct DirectArgs {
  Geo in, mask, out;
  int cin, cout, cout_pad;
  float out_slope;    // activation slope applied to negative outputs (1 = none)
  float mask_slope;   // multiplies inputs whose mask value is <= 0 (only when MASKED)
  int64_t total;      // n * out.ds * h * w
};

template <typename T, bool MASKED>
__global__ void __launch_bounds__(256) conv3d_direct_kernel(const T* __restrict__ in, const T* __restrict__ mask,
                                                            const float* __restrict__ wk, const float* __restrict__ bias,
                                                            T* __restrict__ out, DirectArgs a) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  const int W = a.out.w, H = a.out.h;
  int v = (int)(t % W); t /= W;
  int h = (int)(t % H); t /= H;
  int ps = (int)(t % a.out.ds);          // stored plane of out
  int n = (int)(t / a.out.ds);
  const int p = ps - a.out.hlo;          // local interior index
  const int co0 = blockIdx.y * COT;
  float acc[COT];
  const int64_t gp = a.out.doff + p;
  const bool inside = gp >= 0 && gp < a.out.dglob;
#pragma unroll
  for (int j = 0; j < COT; ++j) acc[j] = (inside && bias && co0 + j < a.cout) ? bias[co0 + j] : 0.f;
  if (inside) {
    for (int ci = 0; ci < a.cin; ++ci) {
      const T* inc = in + n * a.in.nstride + ci * a.in.cstride;
      const T* mc = MASKED ? mask + n * a.mask.nstride + ci * a.mask.cstride : nullptr;
      for (int kd = 0; kd < 3; ++kd) {
        const int64_t gq = gp + kd - 1;
        if (gq < 0 || gq >= a.in.dglob) continue;
        const int q = p + kd - 1;
        for (int kh = 0; kh < 3; ++kh) {
          const int hh = h + kh - 1;
          if (hh < 0 || hh >= H) continue;
#pragma unroll
          for (int kw = 0; kw < 3; ++kw) {
            const int vv = v + kw - 1;
            float xv = 0.f;
            if (vv >= 0 && vv < W) {
              xv = ld(inc + (int64_t)(q + a.in.hlo) * a.in.plane + (int64_t)hh * W + vv);
              if (MASKED) {
                float m = ld(mc + (int64_t)(q + a.mask.hlo) * a.mask.plane + (int64_t)hh * W + vv);
                if (!(m > 0.f)) xv *= a.mask_slope;
              }
            }
            const float* wr = wk + ((int64_t)ci * 27 + (kd * 9 + kh * 3 + kw)) * a.cout_pad + co0;
#pragma unroll
            for (int j = 0; j < COT; ++j) acc[j] = fmaf(wr[j], xv, acc[j]);
          }
        }
      }
    }
  }
  T* o = out + n * a.out.nstride + (int64_t)ps * a.out.plane + (int64_t)h * W + v;
#pragma unroll
  for (int j = 0; j < COT; ++j) {
    if (co0 + j < a.cout) {
      float r = acc[j];
      if (!(r > 0.f)) r *= a.out_slope;
      st(o + (int64_t)(co0 + j) * a.out.cstride, inside ? r : 0.f);
    }
  }
}

size_t direct_fwd_ws_bytes(int cin_k, int cout_k) { return (size_t)cin_k * 27 * cdiv(cout_k, COT) * COT * sizeof(float); }

// in: activations (fwd) or dz (bwd-data); mask: z or NULL; transpose: bwd-data weight view.
template <typename T>
h3d_status conv3d_direct(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                         h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                         hipStream_t stream) {
  const int cin_k = in->c, cout_k = out->c;                     // kernel-view channel counts
  const int cin = transpose ? cout_k : cin_k, cout = transpose ? cin_k : cout_k;  // weight-tensor view
  const int cout_pad = (int)cdiv(cout_k, COT) * COT;
  if (ws_bytes < direct_fwd_ws_bytes(cin_k, cout_k) || !ws) return fail(handle, H3D_EWORKSPACE, "conv3d: workspace too small");
  DirectArgs a;
  a.in = make_geo(in);
  a.mask = mask ? make_geo(mask) : a.in;
  a.out = make_geo(out);
  a.cin = cin_k; a.cout = cout_k; a.cout_pad = cout_pad;
  a.out_slope = out_slope; a.mask_slope = mask_slope;
  a.total = (int64_t)out->n * a.out.ds * out->h * out->w;
  if (a.total == 0 || cout_k == 0) return H3D_OK;
  int64_t nw = (int64_t)cin_k * 27 * cout_pad;
  if (nw > 0)
    hipLaunchKernelGGL((pack_w_direct_kernel<T>), dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, stream, (const T*)w,
                       (float*)ws, cin, cout, transpose ? 1 : 0, cout_pad);
  int64_t grid = cdiv(a.total, 256);
  if (grid >= ((int64_t)1 << 31) || cout_pad / COT > 65535) return fail(handle, H3D_EINVAL, "conv3d: too many blocks");
  dim3 g((unsigned)grid, (unsigned)(cout_pad / COT));
  if (mask)
    hipLaunchKernelGGL((conv3d_direct_kernel<T, true>), g, dim3(256), 0, stream, (const T*)in->data, (const T*)mask->data,
                       (const float*)ws, bias, (T*)out->data, a);
  else
    hipLaunchKernelGGL((conv3d_direct_kernel<T, false>), g, dim3(256), 0, stream, (const T*)in->data, (const T*)nullptr,
                       (const float*)ws, bias, (T*)out->data, a);
  return launch_status(handle, "conv3d_direct");
}

template h3d_status conv3d_direct<float>(void*, const h3d_tensor*, const h3d_tensor*, const void*, const float*, h3d_tensor*,
                                         bool, float, float, void*, size_t, hipStream_t);
template h3d_status conv3d_direct<bf16_t>(void*, const h3d_tensor*, const h3d_tensor*, const void*, const float*,
                                          h3d_tensor*, bool, float, float, void*, size_t, hipStream_t);

// ------------------------------------------------------------------------------------ backward-filter
constexpr int BF_COT = 4;       // output channels per block
constexpr int BF_THREADS = 256;

struct BfArgs {
  Geo x, dz, z;
  int cin, cout;
  float mask_slope;
  int64_t voxels;        // n*d*h*w interior voxels
  int64_t chunk;         // voxels per chunk
  int nchunks;
};

// partial layout: [chunk][cout_pad4][cin][28]  (index 27 = bias partial, only meaningful for ci == 0)
template <typename T, bool MASKED>
__global__ void __launch_bounds__(BF_THREADS) bwd_filter_direct_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                                       const T* __restrict__ z, float* __restrict__ part,
                                                                       BfArgs a) {
  const int chunk = blockIdx.x, cog = blockIdx.y, ci = blockIdx.z;
  const int co0 = cog * BF_COT;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  float acc[BF_COT][28];
#pragma unroll
  for (int j = 0; j < BF_COT; ++j)
#pragma unroll
    for (int t = 0; t < 28; ++t) acc[j][t] = 0.f;
  const int64_t v0 = (int64_t)chunk * a.chunk;
  const int64_t v1 = min(v0 + a.chunk, a.voxels);
  for (int64_t vox = v0 + threadIdx.x; vox < v1; vox += BF_THREADS) {
    int64_t r = vox;
    int v = (int)(r % W); r /= W;
    int h = (int)(r % H); r /= H;
    int p = (int)(r % D);
    int n = (int)(r / D);
    float g[BF_COT];
#pragma unroll
    for (int j = 0; j < BF_COT; ++j) {
      g[j] = 0.f;
      if (co0 + j < a.cout) {
        g[j] = ld(dz + n * a.dz.nstride + (co0 + j) * a.dz.cstride + (int64_t)(p + a.dz.hlo) * a.dz.plane + (int64_t)h * W + v);
        if (MASKED) {
          float m = ld(z + n * a.z.nstride + (co0 + j) * a.z.cstride + (int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)h * W + v);
          if (!(m > 0.f)) g[j] *= a.mask_slope;
        }
      }
    }
    const T* xc = x + n * a.x.nstride + ci * a.x.cstride;
    const int64_t gp = a.x.doff + p;
#pragma unroll
    for (int kd = 0; kd < 3; ++kd) {
      const int64_t gq = gp + kd - 1;
      const bool dok = gq >= 0 && gq < a.x.dglob;
#pragma unroll
      for (int kh = 0; kh < 3; ++kh) {
        const int hh = h + kh - 1;
        const bool hok = dok && hh >= 0 && hh < H;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const int vv = v + kw - 1;
          float xv = 0.f;
          if (hok && vv >= 0 && vv < W) xv = ld(xc + (int64_t)(p + kd - 1 + a.x.hlo) * a.x.plane + (int64_t)hh * W + vv);
#pragma unroll
          for (int j = 0; j < BF_COT; ++j) acc[j][kd * 9 + kh * 3 + kw] = fmaf(g[j], xv, acc[j][kd * 9 + kh * 3 + kw]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < BF_COT; ++j) acc[j][27] += g[j];
  }
  // fixed-shape reduction: butterfly inside each wavefront, then the four wavefronts in order
  __shared__ float red[BF_THREADS / 64][BF_COT * 28];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < BF_COT; ++j)
#pragma unroll
    for (int t = 0; t < 28; ++t) {
      float s = acc[j][t];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0) red[wave][j * 28 + t] = s;
    }
  __syncthreads();
  if (threadIdx.x < BF_COT * 28) {
    float s = red[0][threadIdx.x];
    for (int wv = 1; wv < BF_THREADS / 64; ++wv) s += red[wv][threadIdx.x];
    int j = threadIdx.x / 28, t = threadIdx.x % 28;
    int cout_pad = gridDim.y * BF_COT;
    part[(((int64_t)chunk * cout_pad + co0 + j) * a.cin + ci) * 28 + t] = s;
  }
}

// dw[co][ci][t] = sum over chunks in order; db[co] from slot 27 of ci == 0
__global__ void bwd_filter_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, float* __restrict__ db,
                                         int cin, int cout, int cout_pad, int nchunks) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t total = (int64_t)cout * cin * 28;
  if (i >= total) return;
  int t = (int)(i % 28);
  int ci = (int)((i / 28) % cin);
  int co = (int)(i / (28 * (int64_t)cin));
  float s = 0.f;
  for (int c = 0; c < nchunks; ++c) s += part[(((int64_t)c * cout_pad + co) * cin + ci) * 28 + t];
  if (t < 27)
    dw[((int64_t)co * cin + ci) * 27 + t] = s;
  else if (ci == 0 && db)
    db[co] = s;
}

static void bf_plan(int64_t voxels, int cin, int cout, int64_t* chunk, int* nchunks) {
  int64_t cout_pad = cdiv(cout, BF_COT) * BF_COT;
  int64_t per_chunk_bytes = cout_pad * cin * 28 * 4;
  int64_t max_chunks = std::max<int64_t>(1, ((int64_t)256 << 20) / std::max<int64_t>(per_chunk_bytes, 1));
  int64_t want = std::min<int64_t>(std::min<int64_t>(1024, max_chunks), std::max<int64_t>(1, cdiv(voxels, 2048)));
  *chunk = std::max<int64_t>(1, cdiv(voxels, want));
  *nchunks = (int)std::max<int64_t>(1, cdiv(voxels, *chunk));
}

size_t direct_bf_ws_bytes(const h3d_tensor* x, int cout) {
  int64_t voxels = (int64_t)x->n * x->d * x->h * x->w, chunk;
  int nchunks;
  bf_plan(voxels, x->c, cout, &chunk, &nchunks);
  return (size_t)nchunks * cdiv(cout, BF_COT) * BF_COT * x->c * 28 * sizeof(float);
}

template <typename T>
h3d_status bwd_filter_direct(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                             float* db, float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  BfArgs a;
  a.x = make_geo(x); a.dz = make_geo(dz); a.z = z ? make_geo(z) : a.dz;
  a.cin = x->c; a.cout = dz->c; a.mask_slope = mask_slope;
  a.voxels = (int64_t)x->n * x->d * x->h * x->w;
  if (a.cin == 0 || a.cout == 0) return H3D_OK;
  bf_plan(a.voxels, a.cin, a.cout, &a.chunk, &a.nchunks);
  if (!ws || ws_bytes < direct_bf_ws_bytes(x, a.cout)) return fail(handle, H3D_EWORKSPACE, "conv3d_bwd_filter: workspace too small");
  int cog = (int)cdiv(a.cout, BF_COT);
  if (cog > 65535 || a.cin > 65535) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: too many channels");
  dim3 g((unsigned)a.nchunks, (unsigned)cog, (unsigned)a.cin);
  if (z)
    hipLaunchKernelGGL((bwd_filter_direct_kernel<T, true>), g, dim3(BF_THREADS), 0, stream, (const T*)x->data,
                       (const T*)dz->data, (const T*)z->data, (float*)ws, a);
  else
    hipLaunchKernelGGL((bwd_filter_direct_kernel<T, false>), g, dim3(BF_THREADS), 0, stream, (const T*)x->data,
                       (const T*)dz->data, (const T*)nullptr, (float*)ws, a);
  int64_t total = (int64_t)a.cout * a.cin * 28;
  hipLaunchKernelGGL(bwd_filter_reduce_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, stream, (const float*)ws, dw,
                     db, a.cin, a.cout, cog * BF_COT, a.nchunks);
  return launch_status(handle, "conv3d_bwd_filter_direct");
}

template h3d_status bwd_filter_direct<float>(void*, const h3d_tensor*, const h3d_tensor*, const h3d_tensor*, float*, float*,
                                             float, void*, size_t, hipStream_t);
template h3d_status bwd_filter_direct<bf16_t>(void*, const h3d_tensor*, const h3d_tensor*, const h3d_tensor*, float*, float*,
                                              float, void*, size_t, hipStream_t);

}  // namespace h3d
