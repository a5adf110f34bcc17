// Supporting layers of the two network shapes: 2x2x2 stride-2 transposed convolution (U-Net
// up-sampling), fully-connected layers and the MSE loss (CosmoFlow head).  These are general
// direct kernels with fp32 accumulation; the deconvolution is HBM-bound at U-Net shapes (one tap
// per output voxel), the dense layers are weight-streaming GEMVs (m <= 8 rows).
#include <algorithm>

#include "common.h"

namespace h3d {

// ------------------------------------------------------------------ deconv 2x2x2 stride 2
constexpr int DC_COT = 8;

// w [cin][cout][8] (T) -> fwd: wk fp32 [cin][cout_pad][8];  bwd-data: wk fp32 [cout][8][cin_pad]
template <typename T>
__global__ void deconv_pack_kernel(const T* __restrict__ w, float* __restrict__ wk, int cin, int cout, int pad, int mode) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (mode == 0) {
    int64_t total = (int64_t)cin * pad * 8;
    if (i >= total) return;
    int k = (int)(i % 8), co = (int)((i / 8) % pad), ci = (int)(i / (8 * (int64_t)pad));
    wk[i] = co < cout ? ld(&w[((int64_t)ci * cout + co) * 8 + k]) : 0.f;
  } else {
    int64_t total = (int64_t)cout * 8 * pad;
    if (i >= total) return;
    int ci = (int)(i % pad), k = (int)((i / pad) % 8), co = (int)(i / (8 * (int64_t)pad));
    wk[i] = ci < cin ? ld(&w[((int64_t)ci * cout + co) * 8 + k]) : 0.f;
  }
}

struct DcArgs {
  Geo x, y;          // x: coarse tensor, y: fine tensor (2x)
  int cin, cout, pad;
  int64_t total;     // n * x.d * x.h * x.w
};

template <typename T>
__global__ void __launch_bounds__(256) deconv_fwd_kernel(const T* __restrict__ x, const float* __restrict__ wk,
                                                         const float* __restrict__ bias, T* __restrict__ y, DcArgs a) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int v = (int)(t % a.x.w); t /= a.x.w;
  int h = (int)(t % a.x.h); t /= a.x.h;
  int q = (int)(t % a.x.d);
  int n = (int)(t / a.x.d);
  const int co0 = blockIdx.y * DC_COT;
  float acc[DC_COT][8];
#pragma unroll
  for (int j = 0; j < DC_COT; ++j) {
    float b = (bias && co0 + j < a.cout) ? bias[co0 + j] : 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[j][k] = b;
  }
  const T* xp = x + n * a.x.nstride + (int64_t)(q + a.x.hlo) * a.x.plane + (int64_t)h * a.x.w + v;
  for (int ci = 0; ci < a.cin; ++ci) {
    float xv = ld(xp + ci * a.x.cstride);
    const float* wr = wk + ((int64_t)ci * a.pad + co0) * 8;
#pragma unroll
    for (int j = 0; j < DC_COT; ++j)
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[j][k] = fmaf(wr[j * 8 + k], xv, acc[j][k]);
  }
#pragma unroll
  for (int j = 0; j < DC_COT; ++j) {
    if (co0 + j >= a.cout) continue;
    T* yp = y + n * a.y.nstride + (co0 + j) * a.y.cstride + (int64_t)(2 * q + a.y.hlo) * a.y.plane + (int64_t)(2 * h) * a.y.w + 2 * v;
#pragma unroll
    for (int k = 0; k < 8; ++k) st(yp + (k >> 2) * a.y.plane + ((k >> 1) & 1) * a.y.w + (k & 1), acc[j][k]);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) deconv_bwd_data_kernel(const T* __restrict__ dy, const float* __restrict__ wk,
                                                              T* __restrict__ dx, DcArgs a) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.total) return;
  int v = (int)(t % a.x.w); t /= a.x.w;
  int h = (int)(t % a.x.h); t /= a.x.h;
  int q = (int)(t % a.x.d);
  int n = (int)(t / a.x.d);
  const int ci0 = blockIdx.y * DC_COT;
  float acc[DC_COT];
#pragma unroll
  for (int j = 0; j < DC_COT; ++j) acc[j] = 0.f;
  const T* yp0 = dy + n * a.y.nstride + (int64_t)(2 * q + a.y.hlo) * a.y.plane + (int64_t)(2 * h) * a.y.w + 2 * v;
  for (int co = 0; co < a.cout; ++co) {
    const T* yp = yp0 + co * a.y.cstride;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float g = ld(yp + (k >> 2) * a.y.plane + ((k >> 1) & 1) * a.y.w + (k & 1));
      const float* wr = wk + ((int64_t)co * 8 + k) * a.pad + ci0;
#pragma unroll
      for (int j = 0; j < DC_COT; ++j) acc[j] = fmaf(wr[j], g, acc[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < DC_COT; ++j)
    if (ci0 + j < a.cin)
      st(dx + n * a.x.nstride + (ci0 + j) * a.x.cstride + (int64_t)(q + a.x.hlo) * a.x.plane + (int64_t)h * a.x.w + v, acc[j]);
}

constexpr int DF_COT = 4;
struct DfArgs {
  Geo x, y;
  int cin, cout;
  int64_t voxels, chunk;
  int nchunks;
};

// partial [chunk][cout_pad4][cin][9]  (slot 8 = bias partial, meaningful for ci == 0)
template <typename T>
__global__ void __launch_bounds__(256) deconv_bwd_filter_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                                float* __restrict__ part, DfArgs a) {
  const int chunk = blockIdx.x, co0 = blockIdx.y * DF_COT, ci = blockIdx.z;
  float acc[DF_COT][9];
#pragma unroll
  for (int j = 0; j < DF_COT; ++j)
#pragma unroll
    for (int k = 0; k < 9; ++k) acc[j][k] = 0.f;
  const int64_t v0 = (int64_t)chunk * a.chunk, v1 = min(v0 + a.chunk, a.voxels);
  for (int64_t vox = v0 + threadIdx.x; vox < v1; vox += 256) {
    int64_t r = vox;
    int v = (int)(r % a.x.w); r /= a.x.w;
    int h = (int)(r % a.x.h); r /= a.x.h;
    int q = (int)(r % a.x.d);
    int n = (int)(r / a.x.d);
    float xv = ld(x + n * a.x.nstride + ci * a.x.cstride + (int64_t)(q + a.x.hlo) * a.x.plane + (int64_t)h * a.x.w + v);
#pragma unroll
    for (int j = 0; j < DF_COT; ++j) {
      if (co0 + j >= a.cout) continue;
      const T* yp = dy + n * a.y.nstride + (co0 + j) * a.y.cstride + (int64_t)(2 * q + a.y.hlo) * a.y.plane +
                    (int64_t)(2 * h) * a.y.w + 2 * v;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float g = ld(yp + (k >> 2) * a.y.plane + ((k >> 1) & 1) * a.y.w + (k & 1));
        acc[j][k] = fmaf(xv, g, acc[j][k]);
        acc[j][8] += g;
      }
    }
  }
  __shared__ float red[4][DF_COT * 9];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < DF_COT; ++j)
#pragma unroll
    for (int k = 0; k < 9; ++k) {
      float s = acc[j][k];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0) red[wave][j * 9 + k] = s;
    }
  __syncthreads();
  if (threadIdx.x < DF_COT * 9) {
    float s = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
    int j = threadIdx.x / 9, k = threadIdx.x % 9;
    int cout_pad = gridDim.y * DF_COT;
    part[(((int64_t)chunk * cout_pad + co0 + j) * a.cin + ci) * 9 + k] = s;
  }
}

__global__ void deconv_bf_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, float* __restrict__ db, int cin,
                                        int cout, int cout_pad, int nchunks) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)cout * cin * 9) return;
  int k = (int)(i % 9), ci = (int)((i / 9) % cin), co = (int)(i / (9 * (int64_t)cin));
  float s = 0.f;
  for (int c = 0; c < nchunks; ++c) s += part[(((int64_t)c * cout_pad + co) * cin + ci) * 9 + k];
  if (k < 8)
    dw[((int64_t)ci * cout + co) * 8 + k] = s;
  else if (ci == 0 && db)
    db[co] = s;
}

static void df_plan(int64_t voxels, int cin, int cout, int64_t* chunk, int* nchunks) {
  int64_t per = cdiv(cout, DF_COT) * DF_COT * (int64_t)cin * 9 * 4;
  int64_t maxc = std::max<int64_t>(1, ((int64_t)128 << 20) / std::max<int64_t>(per, 1));
  int64_t want = std::min<int64_t>(std::min<int64_t>(512, maxc), std::max<int64_t>(1, cdiv(voxels, 2048)));
  *chunk = std::max<int64_t>(1, cdiv(voxels, want));
  *nchunks = (int)std::max<int64_t>(1, cdiv(voxels, *chunk));
}

static h3d_status deconv_check(void* handle, const h3d_tensor* x, const h3d_tensor* y, const char* what) {
  H3D_TRY(check_tensor(handle, x, "x"));
  H3D_TRY(check_tensor(handle, y, "y"));
  if (x->dtype != y->dtype || x->n != y->n || y->d != 2 * x->d || y->h != 2 * x->h || y->w != 2 * x->w ||
      y->d_offset != 2 * x->d_offset || y->d_global != 2 * x->d_global)
    return fail(handle, H3D_EINVAL, "%s: fine tensor must be exactly twice the coarse one (extents and offsets)", what);
  return H3D_OK;
}

// ------------------------------------------------------------------ dense (m <= 8) and MSE
constexpr int DM = 8;

struct DenseArgs {
  int m, n, k;
  float slope;
  int act;
};

template <typename T>
__global__ void __launch_bounds__(256) dense_fwd_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                        const float* __restrict__ bias, T* __restrict__ y, DenseArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + wave;
  if (j >= a.n) return;
  float acc[DM];
#pragma unroll
  for (int i = 0; i < DM; ++i) acc[i] = 0.f;
  const T* wr = w + (int64_t)j * a.k;
  constexpr int V = 16 / sizeof(T);
  const bool vec = (a.k % V == 0) && ((uintptr_t)w % 16 == 0) && ((uintptr_t)x % 16 == 0);
  if (vec) {
    struct alignas(16) Pk { T v[V]; };
    constexpr int UN = sizeof(T) == 2 ? 8 : 4;   // weight loads in flight per lane
    for (int k0 = lane * V; k0 < a.k; k0 += 64 * V * UN) {
      Pk wv[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int kk = k0 + u * 64 * V;
        if (kk < a.k) wv[u] = *reinterpret_cast<const Pk*>(wr + kk);
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int kk = k0 + u * 64 * V;
        if (kk < a.k) {
#pragma unroll
          for (int i = 0; i < DM; ++i) {
            if (i < a.m) {
              Pk xv = *reinterpret_cast<const Pk*>(x + (int64_t)i * a.k + kk);
#pragma unroll
              for (int e = 0; e < V; ++e) acc[i] = fmaf(ld(&wv[u].v[e]), ld(&xv.v[e]), acc[i]);
            }
          }
        }
      }
    }
  } else {
    for (int k0 = lane; k0 < a.k; k0 += 64) {
      float wv = ld(wr + k0);
#pragma unroll
      for (int i = 0; i < DM; ++i)
        if (i < a.m) acc[i] = fmaf(wv, ld(x + (int64_t)i * a.k + k0), acc[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < DM; ++i) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (lane == 0) {
    float b = bias ? bias[j] : 0.f;
#pragma unroll
    for (int i = 0; i < DM; ++i)
      if (i < a.m) {
        float r = acc[i] + b;
        if (!(r > 0.f)) r *= a.slope;
        st(y + (int64_t)i * a.n + j, r);
      }
  }
}

// Forward for inputs that fit the LDS (m * k elements <= 128 KB, k a multiple of 16 / sizeof(T)): x is staged once
// per (persistent) workgroup, every weight row is then streamed from HBM exactly once by one wavefront and
// meets x in LDS, so the L2 sees the weights only.  Eight wavefronts per workgroup, rows handed out round-robin.
typedef __bf16 dn_bf16x2 __attribute__((ext_vector_type(2)));
template <typename T>
__global__ void __launch_bounds__(512) dense_fwd_lds_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                            const float* __restrict__ bias, T* __restrict__ y, DenseArgs a) {
  constexpr int V = 16 / sizeof(T);
  struct alignas(16) Pk { T v[V]; };
  extern __shared__ uint4 x_lds[];      // [m][k / V] units
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ku = a.k / V;
  for (int i = tid; i < a.m * ku; i += 512) x_lds[i] = reinterpret_cast<const uint4*>(x)[i];
  __syncthreads();
  for (int j = blockIdx.x * 8 + wave; j < a.n; j += gridDim.x * 8) {
    float acc[DM];
#pragma unroll
    for (int i = 0; i < DM; ++i) acc[i] = 0.f;
    const uint4* wr = reinterpret_cast<const uint4*>(w + (int64_t)j * a.k);
    constexpr int UN = sizeof(T) == 2 ? 8 : 4;   // weight loads in flight per lane
    for (int u0 = lane; u0 < ku; u0 += 64 * UN) {
      uint4 wv[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u)
        if (u0 + 64 * u < ku) wv[u] = wr[u0 + 64 * u];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int uu = u0 + 64 * u;
        if (uu < ku) {
          const Pk wp = __builtin_bit_cast(Pk, wv[u]);
#pragma unroll
          for (int i = 0; i < DM; ++i) {
            if (i < a.m) {
              if constexpr (sizeof(T) == 2) {
                // bf16: one v_dot2 per pair of weights, no conversions
                const uint4 xq = x_lds[i * ku + uu];
                acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wv[u].x), __builtin_bit_cast(dn_bf16x2, xq.x), acc[i], false);
                acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wv[u].y), __builtin_bit_cast(dn_bf16x2, xq.y), acc[i], false);
                acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wv[u].z), __builtin_bit_cast(dn_bf16x2, xq.z), acc[i], false);
                acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wv[u].w), __builtin_bit_cast(dn_bf16x2, xq.w), acc[i], false);
              } else {
                const Pk xp = __builtin_bit_cast(Pk, x_lds[i * ku + uu]);
#pragma unroll
                for (int e = 0; e < V; ++e) acc[i] = fmaf(ld(&wp.v[e]), ld(&xp.v[e]), acc[i]);
              }
            }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < DM; ++i) {
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) acc[i] += __shfl_xor(acc[i], off, 64);
    }
    if (lane == 0) {
      const float b = bias ? bias[j] : 0.f;
#pragma unroll
      for (int i = 0; i < DM; ++i)
        if (i < a.m) {
          float r = acc[i] + b;
          if (!(r > 0.f)) r *= a.slope;
          st(y + (int64_t)i * a.n + j, r);
        }
    }
  }
}

// Forward for long rows in bf16 with few samples (m <= 4, k = UPL * 4096, UPL <= 4): the whole workgroup reads a weight
// row together, so that every load instruction covers 8 KB of consecutive bytes (a wavefront that walks a row by
// itself leaves the memory system 16 separate streams per CU; measured 27 us against 20 for the bare reads, and 13-15
// for fully coalesced ones).  A lane always meets the same k positions, so its part of x stays in registers for the
// whole kernel and nothing goes through LDS except the row sums: per row a butterfly inside each wavefront, the eight
// wavefront sums added in wavefront order at the end (fixed order: same bits every run).  Workgroup b takes rows
// b, b + G, ...: neighbouring workgroups read neighbouring rows.
constexpr int DR_THREADS = 512, DR_MAXROWS = 16, DR_M = 4;
template <int UPL>
__global__ void __launch_bounds__(DR_THREADS) dense_fwd_rows_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                                    const float* __restrict__ bias, bf16_t* __restrict__ y, DenseArgs a) {
  __shared__ float red[DR_MAXROWS][DR_THREADS / 64][DR_M];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ku = a.k / 8;                       // 16-byte units per row = UPL * 512
  uint4 xr[DR_M][UPL];
#pragma unroll
  for (int i = 0; i < DR_M; ++i)
#pragma unroll
    for (int u = 0; u < UPL; ++u)
      xr[i][u] = i < a.m ? reinterpret_cast<const uint4*>(x + (int64_t)i * a.k)[tid + DR_THREADS * u] : uint4{0, 0, 0, 0};
  const int G = gridDim.x;
  int nrows = 0;
  uint4 wv[2][UPL];
  auto load_row = [&](uint4 (&dst)[UPL], int j) {
    const uint4* wr = reinterpret_cast<const uint4*>(w + (int64_t)j * a.k);
#pragma unroll
    for (int u = 0; u < UPL; ++u) dst[u] = wr[tid + DR_THREADS * u];
  };
  auto row = [&](const uint4 (&wq)[UPL], int slot) {
    float acc[DR_M];
#pragma unroll
    for (int i = 0; i < DR_M; ++i) {
      acc[i] = 0.f;
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wq[u].x), __builtin_bit_cast(dn_bf16x2, xr[i][u].x), acc[i], false);
        acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wq[u].y), __builtin_bit_cast(dn_bf16x2, xr[i][u].y), acc[i], false);
        acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wq[u].z), __builtin_bit_cast(dn_bf16x2, xr[i][u].z), acc[i], false);
        acc[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dn_bf16x2, wq[u].w), __builtin_bit_cast(dn_bf16x2, xr[i][u].w), acc[i], false);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) acc[i] += __shfl_xor(acc[i], off, 64);
    }
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < DR_M; ++i) red[slot][wave][i] = acc[i];
    }
  };
  // rows of this workgroup: j = blockIdx.x + G * r, at most DR_MAXROWS of them (the host sizes the grid accordingly)
  int j = blockIdx.x;
  if (j < a.n) load_row(wv[0], j);
  for (; j < a.n; j += 2 * G) {
    const int j1 = j + G, j2 = j + 2 * G;
    if (j1 < a.n) load_row(wv[1], j1);
    row(wv[0], nrows++);
    if (j1 < a.n) {
      if (j2 < a.n) load_row(wv[0], j2);
      row(wv[1], nrows++);
    }
  }
  __syncthreads();
  if (tid < nrows * DR_M) {
    const int r = tid / DR_M, i = tid % DR_M;
    float s = red[r][0][i];
#pragma unroll
    for (int wv2 = 1; wv2 < DR_THREADS / 64; ++wv2) s += red[r][wv2][i];
    const int jj = blockIdx.x + G * r;
    if (i < a.m) {
      float v = s + (bias ? bias[jj] : 0.f);
      if (!(v > 0.f)) v *= a.slope;
      y[(int64_t)i * a.n + jj] = f32_to_bf16(v);
    }
  }
}

template <typename T>
__device__ __forceinline__ float dense_g(const T* dy, const T* y, int64_t idx, const DenseArgs& a) {
  float g = ld(dy + idx);
  if (a.act != H3D_ACT_NONE && !(ld(y + idx) > 0.f)) g *= a.slope;
  return g;
}

// dx[i][c] = sum_j g[i][j] w[j][c].  Weight-streaming: a block of 1024 threads = 16 wavefronts covers
// 128 columns (two per lane, one 4-byte load for bf16); wavefront r takes rows j = r, r+16, ... with
// four rows in flight per iteration; the 16 partial sums meet in LDS and are added in wavefront order.
template <typename T>
__global__ void __launch_bounds__(1024) dense_bwd_dx_kernel(const T* __restrict__ w, const T* __restrict__ y,
                                                            const T* __restrict__ dy, T* __restrict__ dx, DenseArgs a) {
  constexpr int CW = 2;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c0 = (blockIdx.x * 64 + lane) * CW;
  const bool pair_ok = (a.k % CW == 0) && c0 + CW <= a.k && ((uintptr_t)w % (CW * sizeof(T)) == 0);
  float acc[DM][CW];
#pragma unroll
  for (int i = 0; i < DM; ++i)
#pragma unroll
    for (int e = 0; e < CW; ++e) acc[i][e] = 0.f;
  constexpr int UN = 4;
  for (int j0 = wave; j0 < a.n; j0 += 16 * UN) {
    float wv[UN][CW];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + 16 * u;
#pragma unroll
      for (int e = 0; e < CW; ++e) wv[u][e] = 0.f;
      if (j < a.n) {
        if (pair_ok) {
          struct alignas(CW * sizeof(T)) P2 { T v[CW]; };
          P2 p = *reinterpret_cast<const P2*>(w + (int64_t)j * a.k + c0);
#pragma unroll
          for (int e = 0; e < CW; ++e) wv[u][e] = ld(&p.v[e]);
        } else {
#pragma unroll
          for (int e = 0; e < CW; ++e)
            if (c0 + e < a.k) wv[u][e] = ld(w + (int64_t)j * a.k + c0 + e);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + 16 * u;
      if (j < a.n) {
#pragma unroll
        for (int i = 0; i < DM; ++i)
          if (i < a.m) {
            const float g = dense_g(dy, y, (int64_t)i * a.n + j, a);
#pragma unroll
            for (int e = 0; e < CW; ++e) acc[i][e] = fmaf(g, wv[u][e], acc[i][e]);
          }
      }
    }
  }
  __shared__ float red[16][64 * CW + 1];
  for (int i = 0; i < a.m; ++i) {
#pragma unroll
    for (int e = 0; e < CW; ++e) {
      float s = 0.f;
#pragma unroll
      for (int ii = 0; ii < DM; ++ii)
        if (ii == i) s = acc[ii][e];
      red[wave][lane * CW + e] = s;
    }
    __syncthreads();
    if (threadIdx.x < 64 * CW) {
      float s = 0.f;
      for (int r = 0; r < 16; ++r) s += red[r][threadIdx.x];
      int c = blockIdx.x * 64 * CW + threadIdx.x;
      if (c < a.k) st(dx + (int64_t)i * a.k + c, s);
    }
    __syncthreads();
  }
}

// dx for 16-byte-aligned rows (k a multiple of 16 / sizeof(T)): a block owns 8 lanes' worth of columns
// (8 x 16 bytes = one 128-byte line per weight row) and walks ALL n rows: a wavefront is 8 rows x 8
// lanes, 16 wavefronts take 128 rows per step with four steps in flight, so every weight byte is read
// once, in whole lines, with k / (8 V) blocks in flight.  g = dy (.) act'(y) is staged once in LDS as
// [j][m].  The 8 x 16 partial sums of a column meet in a fixed order (row lanes by butterfly, then
// wavefronts in order), so the result does not depend on scheduling.
template <typename T>
__global__ void __launch_bounds__(1024) dense_bwd_dx_vec_kernel(const T* __restrict__ w, const T* __restrict__ y,
                                                                const T* __restrict__ dy, T* __restrict__ dx, DenseArgs a) {
  constexpr int V = 16 / sizeof(T);
  struct alignas(16) Pk { T v[V]; };
  extern __shared__ float g_lds[];      // [n][DM]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  for (int idx = tid; idx < a.n * DM; idx += 1024) {
    const int j = idx / DM, i = idx % DM;
    g_lds[idx] = i < a.m ? dense_g(dy, y, (int64_t)i * a.n + j, a) : 0.f;
  }
  __syncthreads();
  const int rl = lane >> 3, cl = lane & 7;
  const int c0 = (blockIdx.x * 8 + cl) * V;
  const bool col_ok = c0 < a.k;
  float acc[DM][V];
#pragma unroll
  for (int i = 0; i < DM; ++i)
#pragma unroll
    for (int e = 0; e < V; ++e) acc[i][e] = 0.f;
  constexpr int UN = 4;
  for (int j0 = wave * 8 + rl; j0 < a.n; j0 += 128 * UN) {
    Pk wv[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + 128 * u;
      if (j < a.n && col_ok) wv[u] = *reinterpret_cast<const Pk*>(w + (int64_t)j * a.k + c0);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + 128 * u;
      if (j < a.n && col_ok) {
        const float4 ga = *reinterpret_cast<const float4*>(g_lds + j * DM), gb = *reinterpret_cast<const float4*>(g_lds + j * DM + 4);
        const float gv[DM] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float wf = ld(&wv[u].v[e]);
#pragma unroll
          for (int i = 0; i < DM; ++i) acc[i][e] = fmaf(gv[i], wf, acc[i][e]);
        }
      }
    }
  }
  // rows of the wavefront: butterfly over the row lanes (bits 3..5 of the lane id)
#pragma unroll
  for (int i = 0; i < DM; ++i)
#pragma unroll
    for (int e = 0; e < V; ++e) {
      float v = acc[i][e];
      v += __shfl_xor(v, 8, 64);
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      acc[i][e] = v;
    }
  __syncthreads();                       // g_lds is reused for the wavefront partials: [16][DM][8 V]
  float* red = g_lds;
  if (rl == 0) {
#pragma unroll
    for (int i = 0; i < DM; ++i)
#pragma unroll
      for (int e = 0; e < V; ++e) red[(wave * DM + i) * 8 * V + cl * V + e] = acc[i][e];
  }
  __syncthreads();
  for (int idx = tid; idx < a.m * 8 * V; idx += 1024) {
    const int i = idx / (8 * V), c = idx % (8 * V);
    float s = 0.f;
    for (int r = 0; r < 16; ++r) s += red[(r * DM + i) * 8 * V + c];
    const int col = blockIdx.x * 8 * V + c;
    if (col < a.k) st(dx + (int64_t)i * a.k + col, s);
  }
}

// dw[j][c] = sum_i g[i][j] x[i][c];  db[j] = sum_i g[i][j].  Output-bound (fp32 dw): a thread keeps its four
// columns of x (all m rows) in registers and walks DW_ROWS output rows, one 16-byte store per row.
constexpr int DW_ROWS = 16;
template <typename T>
__global__ void __launch_bounds__(256) dense_bwd_dw_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                           const T* __restrict__ dy, float* __restrict__ dw,
                                                           float* __restrict__ db, DenseArgs a) {
  const int j0 = blockIdx.y * DW_ROWS;
  if (blockIdx.x == 0 && threadIdx.x < DW_ROWS && j0 + threadIdx.x < a.n && db) {
    const int j = j0 + threadIdx.x;
    float s = 0.f;
    for (int i = 0; i < a.m; ++i) s += dense_g(dy, y, (int64_t)i * a.n + j, a);
    db[j] = s;
  }
  const bool vec = (a.k % 4 == 0) && ((uintptr_t)x % (4 * sizeof(T)) == 0) && ((uintptr_t)dw % 16 == 0);
  if (vec) {
    for (int c = (blockIdx.x * 256 + threadIdx.x) * 4; c < a.k; c += gridDim.x * 1024) {
      float xv[DM][4];
#pragma unroll
      for (int i = 0; i < DM; ++i) {
        struct alignas(4 * sizeof(T)) P4 { T v[4]; };
        if (i < a.m) {
          const P4 p = *reinterpret_cast<const P4*>(x + (int64_t)i * a.k + c);
#pragma unroll
          for (int e = 0; e < 4; ++e) xv[i][e] = ld(&p.v[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) xv[i][e] = 0.f;
        }
      }
      for (int jj = 0; jj < DW_ROWS && j0 + jj < a.n; ++jj) {
        const int j = j0 + jj;
        float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < DM; ++i)
          if (i < a.m) {
            const float g = dense_g(dy, y, (int64_t)i * a.n + j, a);     // wave-uniform address: a scalar load
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] = fmaf(g, xv[i][e], s[e]);
          }
        *reinterpret_cast<float4*>(dw + (int64_t)j * a.k + c) = float4{s[0], s[1], s[2], s[3]};
      }
    }
  } else {
    for (int jj = 0; jj < DW_ROWS && j0 + jj < a.n; ++jj) {
      const int j = j0 + jj;
      for (int c = blockIdx.x * 256 + threadIdx.x; c < a.k; c += gridDim.x * 256) {
        float s = 0.f;
        for (int i = 0; i < a.m; ++i) s = fmaf(dense_g(dy, y, (int64_t)i * a.n + j, a), ld(x + (int64_t)i * a.k + c), s);
        dw[(int64_t)j * a.k + c] = s;
      }
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) mse_kernel(const T* __restrict__ pred, const float* __restrict__ target,
                                                  float* __restrict__ loss, T* __restrict__ dpred, int count) {
  float s = 0.f;
  const float inv = 1.f / (float)count;
  for (int i = threadIdx.x; i < count; i += 256) {
    float d = ld(pred + i) - target[i];
    s = fmaf(d, d, s);
    st(dpred + i, 2.f * d * inv);
  }
  __shared__ float red[4];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) loss[0] = (red[0] + red[1] + red[2] + red[3]) * inv;
}

bool deconv_fw_mfma_supported(const h3d_tensor* x, const h3d_tensor* y);
size_t deconv_fw_mfma_ws_bytes(const h3d_tensor* x, const h3d_tensor* y);
h3d_status deconv_fw_mfma(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y, void* ws,
                          size_t ws_bytes, hipStream_t stream);

template <typename T>
static h3d_status deconv_fwd_t(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y, void* ws,
                               size_t ws_bytes, hipStream_t s) {
  DcArgs a;
  a.x = make_geo(x); a.y = make_geo(y); a.cin = x->c; a.cout = y->c;
  a.pad = (int)cdiv(a.cout, DC_COT) * DC_COT;
  a.total = (int64_t)x->n * x->d * x->h * x->w;
  if (a.total == 0 || a.cout == 0) return H3D_OK;
  if (deconv_fw_mfma_supported(x, y)) return deconv_fw_mfma(handle, x, w, bias, y, ws, ws_bytes, s);
  size_t need = (size_t)a.cin * a.pad * 8 * 4;
  if (need && (!ws || ws_bytes < need)) return fail(handle, H3D_EWORKSPACE, "deconv2_fwd: workspace too small");
  if (need) hipLaunchKernelGGL((deconv_pack_kernel<T>), dim3((unsigned)cdiv(need / 4, 256)), dim3(256), 0, s, (const T*)w, (float*)ws, a.cin, a.cout, a.pad, 0);
  dim3 g((unsigned)cdiv(a.total, 256), (unsigned)(a.pad / DC_COT));
  hipLaunchKernelGGL((deconv_fwd_kernel<T>), g, dim3(256), 0, s, (const T*)x->data, (const float*)ws, bias, (T*)y->data, a);
  return launch_status(handle, "deconv2_fwd");
}

bool deconv_bd_mfma_supported(const h3d_tensor* dx, const h3d_tensor* dy, const void* w);
h3d_status deconv_bd_mfma(void* handle, const h3d_tensor* dy, const void* w, h3d_tensor* dx, hipStream_t stream);

template <typename T>
static h3d_status deconv_bwd_data_t(void* handle, const h3d_tensor* dy, const void* w, h3d_tensor* dx, void* ws, size_t ws_bytes,
                                    hipStream_t s) {
  DcArgs a;
  a.x = make_geo(dx); a.y = make_geo(dy); a.cin = dx->c; a.cout = dy->c;
  a.pad = (int)cdiv(a.cin, DC_COT) * DC_COT;
  a.total = (int64_t)dx->n * dx->d * dx->h * dx->w;
  if (a.total == 0 || a.cin == 0) return H3D_OK;
  if (deconv_bd_mfma_supported(dx, dy, w)) return deconv_bd_mfma(handle, dy, w, dx, s);
  size_t need = (size_t)a.cout * 8 * a.pad * 4;
  if (need && (!ws || ws_bytes < need)) return fail(handle, H3D_EWORKSPACE, "deconv2_bwd_data: workspace too small");
  if (need) hipLaunchKernelGGL((deconv_pack_kernel<T>), dim3((unsigned)cdiv(need / 4, 256)), dim3(256), 0, s, (const T*)w, (float*)ws, a.cin, a.cout, a.pad, 1);
  dim3 g((unsigned)cdiv(a.total, 256), (unsigned)(a.pad / DC_COT));
  hipLaunchKernelGGL((deconv_bwd_data_kernel<T>), g, dim3(256), 0, s, (const T*)dy->data, (const float*)ws, (T*)dx->data, a);
  return launch_status(handle, "deconv2_bwd_data");
}

bool deconv_bf_mfma_supported(const h3d_tensor* x, const h3d_tensor* dy);
size_t deconv_bf_mfma_ws_bytes(const h3d_tensor* x, const h3d_tensor* dy);
h3d_status deconv_bf_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dy, float* dw, float* db, void* ws, size_t ws_bytes,
                          hipStream_t stream);

template <typename T>
static h3d_status deconv_bwd_filter_t(void* handle, const h3d_tensor* x, const h3d_tensor* dy, float* dw, float* db, void* ws,
                                      size_t ws_bytes, hipStream_t s) {
  DfArgs a;
  a.x = make_geo(x); a.y = make_geo(dy); a.cin = x->c; a.cout = dy->c;
  a.voxels = (int64_t)x->n * x->d * x->h * x->w;
  if (a.cin == 0 || a.cout == 0) return H3D_OK;
  if (deconv_bf_mfma_supported(x, dy)) return deconv_bf_mfma(handle, x, dy, dw, db, ws, ws_bytes, s);
  df_plan(a.voxels, a.cin, a.cout, &a.chunk, &a.nchunks);
  int cog = (int)cdiv(a.cout, DF_COT);
  size_t need = (size_t)a.nchunks * cog * DF_COT * a.cin * 9 * 4;
  if (!ws || ws_bytes < need) return fail(handle, H3D_EWORKSPACE, "deconv2_bwd_filter: workspace too small");
  if (cog > 65535 || a.cin > 65535) return fail(handle, H3D_EINVAL, "deconv2_bwd_filter: too many channels");
  hipLaunchKernelGGL((deconv_bwd_filter_kernel<T>), dim3((unsigned)a.nchunks, (unsigned)cog, (unsigned)a.cin), dim3(256), 0, s,
                     (const T*)x->data, (const T*)dy->data, (float*)ws, a);
  int64_t total = (int64_t)a.cout * a.cin * 9;
  hipLaunchKernelGGL(deconv_bf_reduce_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, s, (const float*)ws, dw, db, a.cin,
                     a.cout, cog * DF_COT, a.nchunks);
  return launch_status(handle, "deconv2_bwd_filter");
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_deconv2_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* y) {
  if (!handle || !x || !y) return 0;
  size_t b = 0;
  if (op == H3D_OP_FWD) {
    b = (size_t)x->c * cdiv(y->c, DC_COT) * DC_COT * 8 * 4;
    if (deconv_fw_mfma_supported(x, y)) b = std::max(b, deconv_fw_mfma_ws_bytes(x, y));
  }
  else if (op == H3D_OP_BWD_DATA) b = (size_t)y->c * 8 * cdiv(x->c, DC_COT) * DC_COT * 4;
  else if (op == H3D_OP_BWD_FILTER) {
    int64_t chunk; int nchunks;
    df_plan((int64_t)x->n * x->d * x->h * x->w, x->c, y->c, &chunk, &nchunks);
    b = (size_t)nchunks * cdiv(y->c, DF_COT) * DF_COT * x->c * 9 * 4;
    if (deconv_bf_mfma_supported(x, y)) b = std::max(b, deconv_bf_mfma_ws_bytes(x, y));
  }
  return (b + 255) & ~(size_t)255;
}

extern "C" h3d_status h3d_deconv2_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y,
                                      void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(deconv_check(handle, x, y, "deconv2_fwd"));
  if (!w && x->c * y->c > 0) return fail(handle, H3D_EINVAL, "deconv2_fwd: NULL weights");
  return x->dtype == H3D_F32 ? deconv_fwd_t<float>(handle, x, w, bias, y, ws, ws_bytes, (hipStream_t)stream)
                             : deconv_fwd_t<bf16_t>(handle, x, w, bias, y, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" h3d_status h3d_deconv2_bwd_data(void* handle, const h3d_tensor* dy, const void* w, h3d_tensor* dx, void* ws,
                                           size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(deconv_check(handle, dx, dy, "deconv2_bwd_data"));
  if (!w && dx->c * dy->c > 0) return fail(handle, H3D_EINVAL, "deconv2_bwd_data: NULL weights");
  return dx->dtype == H3D_F32 ? deconv_bwd_data_t<float>(handle, dy, w, dx, ws, ws_bytes, (hipStream_t)stream)
                              : deconv_bwd_data_t<bf16_t>(handle, dy, w, dx, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" h3d_status h3d_deconv2_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dy, float* dw, float* db,
                                             void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(deconv_check(handle, x, dy, "deconv2_bwd_filter"));
  if (!dw && x->c * dy->c > 0) return fail(handle, H3D_EINVAL, "deconv2_bwd_filter: NULL dw");
  return x->dtype == H3D_F32 ? deconv_bwd_filter_t<float>(handle, x, dy, dw, db, ws, ws_bytes, (hipStream_t)stream)
                             : deconv_bwd_filter_t<bf16_t>(handle, x, dy, dw, db, ws, ws_bytes, (hipStream_t)stream);
}

static h3d_status dense_check(void* handle, int dtype, int m, int n, int k, int act) {
  if (dtype != H3D_F32 && dtype != H3D_BF16) return fail(handle, H3D_EINVAL, "dense: bad dtype");
  if (m < 0 || n < 0 || k < 0) return fail(handle, H3D_EINVAL, "dense: negative size");
  if (m > DM) return fail(handle, H3D_EUNSUPPORTED, "dense: at most %d rows (samples) per call", DM);
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "dense: bad activation");
  return H3D_OK;
}

extern "C" h3d_status h3d_dense_fwd(void* handle, const void* x, const void* w, const float* bias, void* y, int dtype, int m,
                                    int n, int k, int act, float alpha, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(dense_check(handle, dtype, m, n, k, act));
  if (m == 0 || n == 0) return H3D_OK;
  if (!y || (k > 0 && (!x || !w))) return fail(handle, H3D_EINVAL, "dense_fwd: NULL pointer");
  DenseArgs a{m, n, k, act_slope(act, alpha), act};
  dim3 g((unsigned)cdiv(n, 4));
  // x resident in LDS: whole 16-byte units and at most 128 KB of input
  const int vw = dtype == H3D_F32 ? 4 : 8;
  const size_t x_bytes = (size_t)m * k * (dtype == H3D_F32 ? 4 : 2);
  if (dtype == H3D_BF16 && m <= DR_M && k % 4096 == 0 && k <= 4 * 4096 && n >= 256 && (uintptr_t)x % 16 == 0 && (uintptr_t)w % 16 == 0) {
    const int num_cu = static_cast<Handle*>(handle)->num_cu;
    const int grid = (int)std::max<int64_t>(std::min<int64_t>(num_cu, n), cdiv(n, DR_MAXROWS));   // at most DR_MAXROWS rows per workgroup
    const bf16_t* xp = (const bf16_t*)x;
    const bf16_t* wp = (const bf16_t*)w;
    hipStream_t st = (hipStream_t)stream;
    switch (k / 4096) {
      case 1: hipLaunchKernelGGL(dense_fwd_rows_kernel<1>, dim3(grid), dim3(DR_THREADS), 0, st, xp, wp, bias, (bf16_t*)y, a); break;
      case 2: hipLaunchKernelGGL(dense_fwd_rows_kernel<2>, dim3(grid), dim3(DR_THREADS), 0, st, xp, wp, bias, (bf16_t*)y, a); break;
      case 3: hipLaunchKernelGGL(dense_fwd_rows_kernel<3>, dim3(grid), dim3(DR_THREADS), 0, st, xp, wp, bias, (bf16_t*)y, a); break;
      default: hipLaunchKernelGGL(dense_fwd_rows_kernel<4>, dim3(grid), dim3(DR_THREADS), 0, st, xp, wp, bias, (bf16_t*)y, a); break;
    }
    return launch_status(handle, "dense_fwd");
  }
  if (k % vw == 0 && (uintptr_t)x % 16 == 0 && (uintptr_t)w % 16 == 0 && x_bytes <= 128 * 1024 && n >= 256) {
    const int num_cu = static_cast<Handle*>(handle)->num_cu;
    dim3 gl((unsigned)std::min<int64_t>(num_cu, cdiv(n, 8)));
    static bool attr_set[2] = {false, false};
    const int di = dtype == H3D_F32 ? 0 : 1;
    if (!attr_set[di]) {
      const void* fn = di == 0 ? reinterpret_cast<const void*>(dense_fwd_lds_kernel<float>) : reinterpret_cast<const void*>(dense_fwd_lds_kernel<bf16_t>);
      if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess)
        return fail(handle, H3D_EHIP, "dense_fwd: cannot raise the dynamic LDS limit");
      attr_set[di] = true;
    }
    if (dtype == H3D_F32)
      hipLaunchKernelGGL((dense_fwd_lds_kernel<float>), gl, dim3(512), x_bytes, (hipStream_t)stream, (const float*)x, (const float*)w, bias, (float*)y, a);
    else
      hipLaunchKernelGGL((dense_fwd_lds_kernel<bf16_t>), gl, dim3(512), x_bytes, (hipStream_t)stream, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, a);
    return launch_status(handle, "dense_fwd");
  }
  if (dtype == H3D_F32)
    hipLaunchKernelGGL((dense_fwd_kernel<float>), g, dim3(256), 0, (hipStream_t)stream, (const float*)x, (const float*)w, bias, (float*)y, a);
  else
    hipLaunchKernelGGL((dense_fwd_kernel<bf16_t>), g, dim3(256), 0, (hipStream_t)stream, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, a);
  return launch_status(handle, "dense_fwd");
}

extern "C" h3d_status h3d_dense_bwd(void* handle, const void* x, const void* w, const void* y, const void* dy, void* dx,
                                    float* dw, float* db, int dtype, int m, int n, int k, int act, float alpha, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(dense_check(handle, dtype, m, n, k, act));
  if (n == 0 || k == 0) return H3D_OK;
  if (!x || !w || !dy || (act != H3D_ACT_NONE && !y)) return fail(handle, H3D_EINVAL, "dense_bwd: NULL pointer");
  if (!dw && db) return fail(handle, H3D_EINVAL, "dense_bwd: db is computed together with dw");
  if (!dw && !dx) return H3D_OK;
  DenseArgs a{m, n, k, act_slope(act, alpha), act};
  hipStream_t s = (hipStream_t)stream;
  dim3 gdx((unsigned)cdiv(k, 128)), gdw((unsigned)std::min<int64_t>(cdiv(k, 1024), 64), (unsigned)cdiv(n, DW_ROWS));
  if (n > 65535) return fail(handle, H3D_EINVAL, "dense_bwd: n too large");
  // line-wide dx kernel: whole 16-byte units per row and g (n x 8 floats) within 64 KB of LDS
  const int vw = dtype == H3D_F32 ? 4 : 8;
  const size_t dx_lds = std::max<size_t>((size_t)n * DM * sizeof(float), (size_t)16 * DM * 8 * vw * sizeof(float));
  const bool dx_vec = dx && k % vw == 0 && (uintptr_t)w % 16 == 0 && dx_lds <= 65536;
  if (dtype == H3D_F32) {
    if (dx && dx_vec) hipLaunchKernelGGL((dense_bwd_dx_vec_kernel<float>), dim3((unsigned)cdiv(k, 32)), dim3(1024), dx_lds, s, (const float*)w, (const float*)y, (const float*)dy, (float*)dx, a);
    else if (dx) hipLaunchKernelGGL((dense_bwd_dx_kernel<float>), gdx, dim3(1024), 0, s, (const float*)w, (const float*)y, (const float*)dy, (float*)dx, a);
    if (dw) hipLaunchKernelGGL((dense_bwd_dw_kernel<float>), gdw, dim3(256), 0, s, (const float*)x, (const float*)y, (const float*)dy, dw, db, a);
  } else {
    if (dx && dx_vec) hipLaunchKernelGGL((dense_bwd_dx_vec_kernel<bf16_t>), dim3((unsigned)cdiv(k, 64)), dim3(1024), dx_lds, s, (const bf16_t*)w, (const bf16_t*)y, (const bf16_t*)dy, (bf16_t*)dx, a);
    else if (dx) hipLaunchKernelGGL((dense_bwd_dx_kernel<bf16_t>), gdx, dim3(1024), 0, s, (const bf16_t*)w, (const bf16_t*)y, (const bf16_t*)dy, (bf16_t*)dx, a);
    if (dw) hipLaunchKernelGGL((dense_bwd_dw_kernel<bf16_t>), gdw, dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)y, (const bf16_t*)dy, dw, db, a);
  }
  return launch_status(handle, "dense_bwd");
}

extern "C" h3d_status h3d_mse_fwd_bwd(void* handle, const void* pred, const float* target, float* loss, void* dpred, int dtype,
                                      int count, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (dtype != H3D_F32 && dtype != H3D_BF16) return fail(handle, H3D_EINVAL, "mse: bad dtype");
  if (count <= 0 || count > 65536) return fail(handle, H3D_EINVAL, "mse: count must be in [1, 65536]");
  if (!pred || !target || !loss || !dpred) return fail(handle, H3D_EINVAL, "mse: NULL pointer");
  if (dtype == H3D_F32)
    hipLaunchKernelGGL((mse_kernel<float>), dim3(1), dim3(256), 0, (hipStream_t)stream, (const float*)pred, target, loss, (float*)dpred, count);
  else
    hipLaunchKernelGGL((mse_kernel<bf16_t>), dim3(1), dim3(256), 0, (hipStream_t)stream, (const bf16_t*)pred, target, loss, (bf16_t*)dpred, count);
  return launch_status(handle, "mse_fwd_bwd");
}
