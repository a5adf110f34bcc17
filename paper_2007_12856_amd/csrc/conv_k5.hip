// 5x5x5 convolution, stride 1, two zero voxels of padding (Sec. III-A: the two filter sizes the halo packing is
// specialised for are 3^3 and 5^3; the halo is two planes wide here).  All three passes on a depth shard.
//
// Direct form on the vector ALU with fp32 accumulation (fp32 or bf16 storage):
//   forward / backward-data: a workgroup owns an 8 x 32 tile of one output plane and 16 output channels; per
//     input channel the 5 x 12 x 36 input patch is staged in LDS (zero where the volume ends), every thread owns
//     one voxel and 16 accumulators, and the 125 x 16 weights of the step come as fp32 from a packed copy whose
//     addresses are the same for the whole workgroup (scalar loads, no LDS traffic).  Backward-data is the same
//     kernel on g = dz * act'(z) (mask applied while staging) with the filter reversed and transposed.
//     With bf16 storage the same two passes run on the matrix cores instead (k5_mfma_kernel): v_mfma_f32_32x32x16_bf16
//     with 32 output channels on the rows, 32 voxels of an output row on the columns and 16 input channels of one tap
//     as K; a workgroup owns 16 rows x 32 columns of one output plane, a wavefront 4 of the rows (4 accumulators share
//     every weight fragment, and the 8 patch rows they read per kw feed 20 products); per (16-channel chunk, kd) the
//     20 x 36 input patch of that plane is transposed into LDS channel-innermost (32 bytes per voxel: one 16-byte read
//     per lane is a B fragment at any of the 25 shifts), the weight fragments of the stage come from a packed bf16
//     copy [co block][ci chunk][tap][32 co][16 ci] and pass through LDS with the patch.  The bf16 backward passes
//     make g = dz * act'(z) once (k5_grad_kernel, into the workspace) instead of masking while staging.
//   backward-filter: a workgroup owns (chunk of tiles, ci, 16 output channels); a thread owns one of the 125 taps
//     and 8 of the 16 channels and walks the 256 voxels of a tile with x and g in LDS; per-chunk partial sums go
//     to the workspace and a second kernel adds them in chunk order (two calls give identical bits).  With bf16
//     storage, W a multiple of 8 and 16-byte aligned tensors the partial sums come from k5_bwf_mfma_kernel instead
//     (described above it).
#include "common.h"

namespace h3d {
namespace {

constexpr int K5_TAPS = 125;
constexpr int K5_TH = 8, K5_TW = 32, K5_COB = 16;
constexpr int K5_PH = K5_TH + 4, K5_PW = K5_TW + 4, K5_PWP = K5_PW + 1;
constexpr int K5_PATCH = 5 * K5_PH * K5_PW;

struct K5Args {
  Geo in, out, zg;     // staged tensor (x or dz), written tensor (z or dx), mask tensor (saved output, backward only)
  int pmin, pmax;      // local planes of `in` that are stored and inside the volume: [pmin, pmax)
  int tiles_w, tiles_h, cobs;
  float slope_in;      // factor on staged values where the saved output is not positive
  float slope_out;     // activation of the written values
};

// wp[cob][cl][t][16] fp32, cl the channel the kernels loop over, 16 the channels a thread accumulates.
// forward: wp[cob][ci][t][c] = w[16 cob + c][ci][t];  backward-data: wp[cib][co][t][c] = w[co][16 cib + c][124 - t].
template <typename T>
__global__ void __launch_bounds__(256) k5_pack_w_kernel(const T* __restrict__ w, float* __restrict__ wp, int cin, int cout,
                                                        int transposed, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % K5_COB), t = (int)((i / K5_COB) % K5_TAPS);
  const int loopc = transposed ? cout : cin, accc = transposed ? cin : cout;
  const int cl = (int)((i / (K5_COB * K5_TAPS)) % loopc), cb = (int)(i / ((int64_t)K5_COB * K5_TAPS * loopc));
  const int ca = cb * K5_COB + c;
  float v = 0.f;
  if (ca < accc) {
    const int co = transposed ? cl : ca, ci = transposed ? ca : cl, tt = transposed ? K5_TAPS - 1 - t : t;
    v = ld(w + ((int64_t)co * cin + ci) * K5_TAPS + tt);
  }
  wp[i] = v;
}

// one staged patch value: plane pp (local index), row hh, column ww of channel c of sample n; zero outside
template <typename T, bool MASK>
__device__ __forceinline__ float k5_fetch(const T* __restrict__ in, const T* __restrict__ zm, const K5Args& a, int n, int c, int pp,
                                          int hh, int ww) {
  if (pp < a.pmin || pp >= a.pmax || hh < 0 || hh >= a.in.h || ww < 0 || ww >= a.in.w) return 0.f;
  const int64_t sp = (int64_t)hh * a.in.w + ww;
  float v = ld(in + (int64_t)n * a.in.nstride + (int64_t)c * a.in.cstride + (int64_t)(pp + a.in.hlo) * a.in.plane + sp);
  if (MASK) {
    const float zv = ld(zm + (int64_t)n * a.zg.nstride + (int64_t)c * a.zg.cstride + (int64_t)(pp + a.zg.hlo) * a.zg.plane + sp);
    if (!(zv > 0.f)) v *= a.slope_in;
  }
  return v;
}

template <typename T, bool MASK>
__global__ void __launch_bounds__(256) k5_conv_kernel(const T* __restrict__ in, const T* __restrict__ zm, const float* __restrict__ wp,
                                                      const float* __restrict__ bias, T* __restrict__ out, K5Args a) {
  __shared__ float xs[5][K5_PH][K5_PWP];
  const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
  const int tw = blockIdx.x % a.tiles_w, th = blockIdx.x / a.tiles_w;
  const int p = blockIdx.y;
  const int n = blockIdx.z / a.cobs, cob = blockIdx.z % a.cobs;
  const int h0 = th * K5_TH, w0 = tw * K5_TW;
  float acc[K5_COB];
#pragma unroll
  for (int c = 0; c < K5_COB; ++c) acc[c] = 0.f;
  const float* wb = wp + (int64_t)cob * a.in.c * (K5_TAPS * K5_COB);
  for (int cl = 0; cl < a.in.c; ++cl) {
    __syncthreads();
    for (int idx = tid; idx < K5_PATCH; idx += 256) {
      const int kd = idx / (K5_PH * K5_PW), r = (idx / K5_PW) % K5_PH, c = idx % K5_PW;
      xs[kd][r][c] = k5_fetch<T, MASK>(in, zm, a, n, cl, p + kd - 2, h0 + r - 2, w0 + c - 2);
    }
    __syncthreads();
    const float* wc = wb + (int64_t)cl * (K5_TAPS * K5_COB);
    for (int kd = 0; kd < 5; ++kd)
      for (int kh = 0; kh < 5; ++kh) {
        const float* wr = wc + (kd * 5 + kh) * 5 * K5_COB;
#pragma unroll
        for (int kw = 0; kw < 5; ++kw) {
          const float xv = xs[kd][ty + kh][tx + kw];
#pragma unroll
          for (int c = 0; c < K5_COB; ++c) acc[c] = fmaf(xv, wr[kw * K5_COB + c], acc[c]);
        }
      }
  }
  const int hh = h0 + ty, ww = w0 + tx;
  if (hh >= a.out.h || ww >= a.out.w) return;
  T* o = out + (int64_t)n * a.out.nstride + (int64_t)(p + a.out.hlo) * a.out.plane + (int64_t)hh * a.out.w + ww;
#pragma unroll
  for (int c = 0; c < K5_COB; ++c) {
    const int co = cob * K5_COB + c;
    if (co < a.out.c) {
      float v = acc[c] + (bias ? bias[co] : 0.f);
      if (!(v > 0.f)) v *= a.slope_out;
      st(o + (int64_t)co * a.out.cstride, v);
    }
  }
}

// a.in = x, a.out = dz (the gradient), a.zg = saved output.  grid (chunks, cin, cobs).
// part: [chunk][cout][cin][125], part_db: [chunk][cout]
template <typename T, bool MASK>
__global__ void __launch_bounds__(256) k5_bwf_kernel(const T* __restrict__ x, const T* __restrict__ dz, const T* __restrict__ zm,
                                                     float* __restrict__ part, float* __restrict__ part_db, K5Args a,
                                                     int tiles_total, int tiles_per_chunk) {
  __shared__ float xs[5][K5_PH][K5_PWP];
  __shared__ __attribute__((aligned(16))) float gs[K5_TH * K5_TW][K5_COB];
  const int tid = threadIdx.x;
  const int chunk = blockIdx.x, ci = blockIdx.y, cob = blockIdx.z;
  const bool tap_thread = tid < 2 * K5_TAPS;
  const int tap = tid % K5_TAPS, half = tid >= K5_TAPS ? 1 : 0;
  const int kd = tap / 25, kh = (tap / 5) % 5, kw = tap % 5;
  const bool db_thread = ci == 0 && tid < K5_COB;
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  float dbacc = 0.f;
  const int t_lo = chunk * tiles_per_chunk;
  const int t_hi = min(t_lo + tiles_per_chunk, tiles_total);
  const int tiles_pl = a.tiles_w * a.tiles_h;
  for (int tile = t_lo; tile < t_hi; ++tile) {
    const int tw = tile % a.tiles_w, th = (tile / a.tiles_w) % a.tiles_h;
    const int p = (tile / tiles_pl) % a.in.d, n = tile / (tiles_pl * a.in.d);
    const int h0 = th * K5_TH, w0 = tw * K5_TW;
    __syncthreads();
    for (int idx = tid; idx < K5_PATCH; idx += 256) {
      const int pd = idx / (K5_PH * K5_PW), r = (idx / K5_PW) % K5_PH, c = idx % K5_PW;
      xs[pd][r][c] = k5_fetch<T, false>(x, nullptr, a, n, ci, p + pd - 2, h0 + r - 2, w0 + c - 2);
    }
    for (int idx = tid; idx < K5_TH * K5_TW * K5_COB; idx += 256) {
      const int c = idx / (K5_TH * K5_TW), v = idx % (K5_TH * K5_TW);
      const int co = cob * K5_COB + c, hh = h0 + (v >> 5), ww = w0 + (v & 31);
      float g = 0.f;
      if (co < a.out.c && hh < a.out.h && ww < a.out.w) {
        const int64_t sp = (int64_t)hh * a.out.w + ww;
        g = ld(dz + (int64_t)n * a.out.nstride + (int64_t)co * a.out.cstride + (int64_t)(p + a.out.hlo) * a.out.plane + sp);
        if (MASK) {
          const float zv = ld(zm + (int64_t)n * a.zg.nstride + (int64_t)co * a.zg.cstride + (int64_t)(p + a.zg.hlo) * a.zg.plane + sp);
          if (!(zv > 0.f)) g *= a.slope_in;
        }
      }
      gs[v][c] = g;
    }
    __syncthreads();
    if (tap_thread) {
      const float* xb = &xs[kd][kh][kw];
      for (int vy = 0; vy < K5_TH; ++vy) {
#pragma unroll 8
        for (int vx = 0; vx < K5_TW; ++vx) {
          const float xv = xb[vy * K5_PWP + vx];
          const float4 ga = *reinterpret_cast<const float4*>(&gs[vy * K5_TW + vx][half * 8]);
          const float4 gb = *reinterpret_cast<const float4*>(&gs[vy * K5_TW + vx][half * 8 + 4]);
          acc[0] = fmaf(xv, ga.x, acc[0]); acc[1] = fmaf(xv, ga.y, acc[1]);
          acc[2] = fmaf(xv, ga.z, acc[2]); acc[3] = fmaf(xv, ga.w, acc[3]);
          acc[4] = fmaf(xv, gb.x, acc[4]); acc[5] = fmaf(xv, gb.y, acc[5]);
          acc[6] = fmaf(xv, gb.z, acc[6]); acc[7] = fmaf(xv, gb.w, acc[7]);
        }
      }
    }
    if (db_thread) {
      float s = 0.f;
      for (int v = 0; v < K5_TH * K5_TW; ++v) s += gs[v][tid];
      dbacc += s;
    }
  }
  if (tap_thread) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int co = cob * K5_COB + half * 8 + c;
      if (co < a.out.c) part[(((int64_t)chunk * a.out.c + co) * a.in.c + ci) * K5_TAPS + tap] = acc[c];
    }
  }
  if (db_thread) {
    const int co = cob * K5_COB + tid;
    if (co < a.out.c) part_db[(int64_t)chunk * a.out.c + co] = dbacc;
  }
}

// out[i] = sum over chunks, in chunk order, of part[chunk][i]
__global__ void __launch_bounds__(256) k5_reduce_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t count, int chunks) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s = 0.f;
  for (int c = 0; c < chunks; ++c) s += part[(int64_t)c * count + i];
  out[i] = s;
}

// ---- matrix-core form of forward / backward-data (bf16 storage) ----
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int KM_TH = 16, KM_TW = 32, KM_PH = KM_TH + 4, KM_PW = KM_TW + 4;
constexpr int KM_COB = 32, KM_CIB = 16;

// wpk[cb][cic][t][c][e] bf16: accumulated channel 32 cb + c, looped channel 16 cic + e (zero past the real counts);
// forward: w[co = acc][ci = loop][t];  backward-data: w[co = loop][ci = acc][124 - t].
__global__ void __launch_bounds__(256) k5_pack_w_mfma_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wpk, int cin, int cout,
                                                             int transposed, int cics, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int e = (int)(i % KM_CIB), c = (int)((i / KM_CIB) % KM_COB), t = (int)((i / (KM_CIB * KM_COB)) % K5_TAPS);
  const int cic = (int)((i / ((int64_t)KM_CIB * KM_COB * K5_TAPS)) % cics), cb = (int)(i / ((int64_t)KM_CIB * KM_COB * K5_TAPS * cics));
  const int ca = cb * KM_COB + c, cl = cic * KM_CIB + e;
  const int loopc = transposed ? cout : cin, accc = transposed ? cin : cout;
  bf16_t v = 0;
  if (ca < accc && cl < loopc) {
    const int co = transposed ? cl : ca, ci = transposed ? ca : cl, tt = transposed ? K5_TAPS - 1 - t : t;
    v = w[((int64_t)co * cin + ci) * K5_TAPS + tt];
  }
  wpk[i] = v;
}

// grid (tiles_w * tiles_h, d, n * cobs) with 16 x 32 tiles and blocks of 32 accumulated channels.  Backward-data passes
// g = dz * act'(z), made once by k5_grad_kernel: staging the mask here cost two loads per value, five times per plane.
__global__ void __launch_bounds__(256) k5_mfma_kernel(const bf16_t* __restrict__ in, const bf16_t* __restrict__ wpk,
                                                      const float* __restrict__ bias, bf16_t* __restrict__ out, K5Args a,
                                                      int cics) {
  __shared__ __attribute__((aligned(16))) bf16_t xs[KM_PH * KM_PW * KM_CIB];
  __shared__ __attribute__((aligned(16))) bf16_t wsm[25 * KM_COB * KM_CIB];   // the 25 weight fragments of the stage
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lc = lane & 31, lh = lane >> 5;
  const int tw = blockIdx.x % a.tiles_w, th = blockIdx.x / a.tiles_w;
  const int p = blockIdx.y;
  const int n = blockIdx.z / a.cobs, cob = blockIdx.z % a.cobs;
  const int h0 = th * KM_TH, w0 = tw * KM_TW;
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  // A stage is one (16-channel chunk, kd) pair.  The values of stage s + 1 are loaded into registers before the
  // multiplications of stage s start and go to LDS after them, so the memory latency hides behind the matrix work.
  constexpr int ROUNDS = (KM_PH * KM_PW + 255) / 256;
  bf16_t raw[ROUNDS][KM_CIB];
  const int stages = cics * 5;
  constexpr int WPIECES = 25 * KM_COB * KM_CIB / 8, WROUNDS = (WPIECES + 255) / 256;   // 16-byte pieces of a stage's weights
  uint4 wq[WROUNDS];
  auto load_stage = [&](int s) {
    const int cic = s / 5, pp = p + s % 5 - 2;
    const bool plane_ok = pp >= a.pmin && pp < a.pmax;
    // the weights travel with the patch and are read from LDS: no memory load stands between the products, so
    // nothing waits for the patch of the next stage before its time
    const bf16_t* wt = wpk + (((int64_t)cob * cics + cic) * K5_TAPS + (s % 5) * 25) * (KM_COB * KM_CIB);
#pragma unroll
    for (int q = 0; q < WROUNDS; ++q) {
      const int idx = tid + 256 * q;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (idx < WPIECES) v = *reinterpret_cast<const uint4*>(wt + idx * 8);
      wq[q] = v;
    }
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
      const int pos = tid + 256 * q;
      const int r = pos / KM_PW, c = pos % KM_PW;
      const int hh = h0 + r - 2, ww = w0 + c - 2;
      const bool ok = plane_ok && pos < KM_PH * KM_PW && hh >= 0 && hh < a.in.h && ww >= 0 && ww < a.in.w;
      const int64_t sp = (int64_t)hh * a.in.w + ww;
      const bf16_t* src = in + (int64_t)n * a.in.nstride + (int64_t)(pp + a.in.hlo) * a.in.plane + sp;
#pragma unroll
      for (int e = 0; e < KM_CIB; ++e) {
        const int ci = cic * KM_CIB + e;
        const bool okc = ok && ci < a.in.c;
        raw[q][e] = okc ? src[(int64_t)ci * a.in.cstride] : (bf16_t)0;
      }
    }
  };
  auto store_stage = [&]() {
#pragma unroll
    for (int q = 0; q < WROUNDS; ++q) {
      const int idx = tid + 256 * q;
      if (idx < WPIECES) *reinterpret_cast<uint4*>(wsm + idx * 8) = wq[q];
    }
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
      const int pos = tid + 256 * q;
      if (pos < KM_PH * KM_PW) {
        uint32_t pk[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) pk[e] = 0u;
#pragma unroll
        for (int e = 0; e < KM_CIB; ++e) {
          pk[e >> 1] |= (uint32_t)raw[q][e] << (16 * (e & 1));
        }
        uint4* dst = reinterpret_cast<uint4*>(xs + pos * KM_CIB);
        dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
      }
    }
  };
  load_stage(0);
  for (int s = 0; s < stages; ++s) {
    __syncthreads();          // the multiplications of the stage before have read the patch
    store_stage();
    __syncthreads();
    if (s + 1 < stages) load_stage(s + 1);
    // the 4 output rows of the wavefront and the 5 kh taps meet 8 patch rows: per kw, 8 fragment reads feed 20 products
    const bf16_t* wl = wsm + lc * KM_CIB + lh * 8;
#pragma unroll 1
    for (int kw = 0; kw < 5; ++kw) {
      bf16x8 B[8];
#pragma unroll
      for (int r = 0; r < 8; ++r)
        B[r] = *reinterpret_cast<const bf16x8*>(xs + ((wave * 4 + r) * KM_PW + lc + kw) * KM_CIB + lh * 8);
#pragma unroll
      for (int kh = 0; kh < 5; ++kh) {
        const bf16x8 A = *reinterpret_cast<const bf16x8*>(wl + (kh * 5 + kw) * (KM_COB * KM_CIB));
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B[i + kh], acc[i], 0, 0, 0);
      }
    }
  }
  // accumulator element r of lane (lc, lh): column = voxel lc, row = channel 8 (r / 4) + 4 lh + r % 4
  const int ww = w0 + lc;
  if (ww >= a.out.w) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int hh = h0 + wave * 4 + i;
    if (hh >= a.out.h) continue;
    bf16_t* o = out + (int64_t)n * a.out.nstride + (int64_t)(p + a.out.hlo) * a.out.plane + (int64_t)hh * a.out.w + ww;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = cob * KM_COB + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (co < a.out.c) {
        float v = acc[i][r] + (bias ? bias[co] : 0.f);
        if (!(v > 0.f)) v *= a.slope_out;
        o[(int64_t)co * a.out.cstride] = f32_to_bf16(v);
      }
    }
  }
}

// ---- matrix-core form of backward-filter (bf16 storage, W a multiple of 8, 16-byte aligned tensors) ----
// dw[co][ci][tap] is a contraction over voxels: rows = 32 output channels (A = g), columns = 32 input channels
// (B = x shifted by the tap), K = 16 consecutive voxels of a row; both operands keep NCDHW (8 consecutive W voxels
// are one 16-byte piece).  A workgroup of five wavefronts owns (chunk of 32 x 128 tiles, kd, 32 co, 32 ci); wavefront
// kh holds the five kw accumulators of its (kd, kh).  It walks down the rows of a tile: per output row the g row and
// one new x row go to LDS (x rows in a ring of five: output row t and tap kh read x row t + kh); for 16 voxels the x
// window of 12 elements is read once (4 + 16 + 4 bytes) and the odd shifts are made from it with v_alignbit.
constexpr int KB_TH = 32, KB_TW = 128, KB_C = 32;
constexpr int KB_XW = 152, KB_GW = 136;          // row pitches (elements): 76 and 68 dwords, conflict-free 16-byte reads
constexpr int KB_XG = KB_XW / 8, KB_GG = KB_TW / 8;
constexpr int KB_THREADS = 320;

// `g` is dz, or dz * act'(z) made once by k5_grad_kernel (every (kd, ci block) workgroup reads it).
__global__ void __launch_bounds__(KB_THREADS) k5_bwf_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g,
                                                                 float* __restrict__ part, float* __restrict__ part_db, K5Args a,
                                                                 int units_total, int units_per_chunk, int cibs) {
  __shared__ __attribute__((aligned(16))) bf16_t xr[5 * KB_C * KB_XW];
  __shared__ __attribute__((aligned(16))) bf16_t gr[KB_C * KB_GW];
  const int tid = threadIdx.x, kh = tid >> 6, lane = tid & 63, lc = lane & 31, lh = lane >> 5;
  const int chunk = blockIdx.x, kd = blockIdx.y;
  const int cob = blockIdx.z / cibs, cib = blockIdx.z % cibs;
  const bool db_wave = kd == 2 && cib == 0 && kh == 2;
  f32x16 acc[5];
#pragma unroll
  for (int k = 0; k < 5; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  float dbacc = 0.f;
  const int tiles_pl = a.tiles_w * a.tiles_h;
  const int u_lo = chunk * units_per_chunk;
  const int u_hi = min(u_lo + units_per_chunk, units_total);
  for (int unit = u_lo; unit < u_hi; ++unit) {
    const int wt = unit % a.tiles_w, ht = (unit / a.tiles_w) % a.tiles_h;
    const int p = (unit / tiles_pl) % a.in.d, n = unit / (tiles_pl * a.in.d);
    const int pp = p + kd - 2;
    if (pp < a.pmin || pp >= a.pmax) continue;   // x is zero on that plane (same decision for the whole workgroup)
    const int h0 = ht * KB_TH, w0 = wt * KB_TW;
    const int rows = min(KB_TH, a.in.h - h0);
    const bf16_t* xb = x + (int64_t)n * a.in.nstride + (int64_t)(pp + a.in.hlo) * a.in.plane;
    const bf16_t* gb = g + (int64_t)n * a.out.nstride + (int64_t)(p + a.out.hlo) * a.out.plane;
    uint4 xq0, xq1, gq0, gq1;
    // x row h0 - 2 + j, columns w0 - 8 .. w0 + 143, as 19 pieces of 8 per channel; piece idx of the row
    auto load_x1 = [&](int j, int idx) -> uint4 {
      const int hh = h0 - 2 + j;
      const int cl = idx / KB_XG, g = idx % KB_XG;
      const int ci = cib * KB_C + cl, col = w0 - 8 + 8 * g;
      const bool ok = idx < KB_C * KB_XG && hh >= 0 && hh < a.in.h && ci < a.in.c && col >= 0 && col < a.in.w;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (ok) v = *reinterpret_cast<const uint4*>(xb + (int64_t)ci * a.in.cstride + (int64_t)hh * a.in.w + col);
      return v;
    };
    auto store_x1 = [&](int j, int idx, const uint4& v) {
      if (idx < KB_C * KB_XG) *reinterpret_cast<uint4*>(xr + ((j % 5) * KB_C + idx / KB_XG) * KB_XW + 8 * (idx % KB_XG)) = v;
    };
    // g row h0 + t, columns w0 .. w0 + 127, 16 pieces per channel
    auto load_g1 = [&](int t, int idx, uint4& gv) {
      const int hh = h0 + t;
      const int cl = idx / KB_GG, gi = idx % KB_GG;
      const int co = cob * KB_C + cl, col = w0 + 8 * gi;
      const bool ok = idx < KB_C * KB_GG && hh < a.out.h && co < a.out.c && col < a.out.w;
      const int64_t sp = (int64_t)hh * a.out.w + col;
      gv = make_uint4(0u, 0u, 0u, 0u);
      if (ok) gv = *reinterpret_cast<const uint4*>(gb + (int64_t)co * a.out.cstride + sp);
    };
    auto store_g1 = [&](int idx, const uint4& v) {
      if (idx < KB_C * KB_GG) *reinterpret_cast<uint4*>(gr + (idx / KB_GG) * KB_GW + 8 * (idx % KB_GG)) = v;
    };
    auto load_x = [&](int j) { xq0 = load_x1(j, tid); xq1 = load_x1(j, tid + KB_THREADS); };
    auto store_x = [&](int j) { store_x1(j, tid, xq0); store_x1(j, tid + KB_THREADS, xq1); };
    auto load_g = [&](int t) { load_g1(t, tid, gq0); load_g1(t, tid + KB_THREADS, gq1); };
    auto store_g = [&]() { store_g1(tid, gq0); store_g1(tid + KB_THREADS, gq1); };
    __syncthreads();                 // the tile before has been multiplied
#pragma unroll 1
    for (int j = 0; j < 4; ++j) {
      load_x(j);
      store_x(j);
    }
    load_x(4);
    load_g(0);
    for (int t = 0; t < rows; ++t) {
      __syncthreads();               // row t - 1 has been multiplied: its oldest x row and the g row are free
      store_x(t + 4);
      store_g();
      __syncthreads();
      if (t + 1 < rows) {            // in flight during the multiplications
        load_x(t + 5);
        load_g(t + 1);
      }
      const bf16_t* xrow = xr + (((t + kh) % 5) * KB_C + lc) * KB_XW;
      const bf16_t* grow = gr + lc * KB_GW;
      const int nks = min(KB_TW / 16, (a.in.w - w0 + 15) / 16);   // steps that hold columns of the volume (the rest is g = 0)
#pragma unroll
      for (int ks = 0; ks < KB_TW / 16; ++ks) {
        if ((ks & 3) == 0 && ks >= nks) break;   // decided per group of four steps: inside a group the reads run ahead of the products
        const int e0 = 16 * ks + 8 * lh;
        const bf16x8 A = *reinterpret_cast<const bf16x8*>(grow + e0);
        const uint4 q = *reinterpret_cast<const uint4*>(xrow + 8 + e0);
        const uint32_t dm = *reinterpret_cast<const uint32_t*>(xrow + 6 + e0);
        const uint32_t dp = *reinterpret_cast<const uint32_t*>(xrow + 16 + e0);
        // dwords dm, q.x .. q.w, dp hold elements -2 .. 9 around the piece; o* are the dwords that start at an odd element
        const uint32_t o0 = __builtin_amdgcn_alignbit(q.x, dm, 16), o1 = __builtin_amdgcn_alignbit(q.y, q.x, 16);
        const uint32_t o2 = __builtin_amdgcn_alignbit(q.z, q.y, 16), o3 = __builtin_amdgcn_alignbit(q.w, q.z, 16);
        const uint32_t o4 = __builtin_amdgcn_alignbit(dp, q.w, 16);
        const uint4 b0 = make_uint4(dm, q.x, q.y, q.z), b1 = make_uint4(o0, o1, o2, o3);
        const uint4 b2 = q, b3 = make_uint4(o1, o2, o3, o4);
        const uint4 b4 = make_uint4(q.y, q.z, q.w, dp);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b0), acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b1), acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b2), acc[2], 0, 0, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b3), acc[3], 0, 0, 0);
        acc[4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b4), acc[4], 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) dbacc += (float)A[e];   // every wavefront sums g (free beside the products); one of them writes it
      }
    }
  }
  // accumulator element r of lane (lc, lh): column = input channel lc, row = output channel 8 (r / 4) + 4 lh + r % 4
  const int ci = cib * KB_C + lc;
#pragma unroll
  for (int kw = 0; kw < 5; ++kw)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = cob * KB_C + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (co < a.out.c && ci < a.in.c)
        part[(((int64_t)chunk * a.out.c + co) * a.in.c + ci) * K5_TAPS + kd * 25 + kh * 5 + kw] = acc[kw][r];
    }
  if (db_wave) {
    const float v = dbacc + __shfl_xor(dbacc, 32, 64);
    const int co = cob * KB_C + lc;
    if (lh == 0 && co < a.out.c) part_db[(int64_t)chunk * a.out.c + co] = v;
  }
}

// g = dz * (z > 0 ? 1 : slope) on every stored plane of dz (bf16), once, so that backward-data stages plain values:
// its workgroups read every plane five times (once per kd) and once per block of output channels.  z may store other
// halo planes than dz; a plane of dz without a stored partner in z is copied (backward-data never reads it).
// One thread per piece of V elements of a plane (V = 8 when planes are whole 16-byte pieces, else 1).
template <int V>
__global__ void __launch_bounds__(256) k5_grad_kernel(const bf16_t* __restrict__ dz, const bf16_t* __restrict__ zm,
                                                      bf16_t* __restrict__ g, Geo dg, Geo zg, float slope, int64_t pieces) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= pieces) return;
  const int64_t per_plane = dg.plane / V;
  const int64_t off = (i % per_plane) * V, sp = (i / per_plane) % dg.ds, nc = i / (per_plane * dg.ds);
  const int64_t di = (nc * dg.ds + sp) * dg.plane + off;
  const int64_t zp = sp - dg.hlo + zg.hlo;
  const bool masked = zp >= 0 && zp < zg.ds;
  const int64_t zi = (nc * zg.ds + zp) * zg.plane + off;
  if (V == 8) {
    uint4 v = *reinterpret_cast<const uint4*>(dz + di);
    if (masked) {
      const uint4 zv = *reinterpret_cast<const uint4*>(zm + zi);
      uint32_t gv[4] = {v.x, v.y, v.z, v.w};
      const uint32_t zz[4] = {zv.x, zv.y, zv.z, zv.w};
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t lo = gv[d] & 0xffffu, hi = gv[d] >> 16;
        if (!(bf16_to_f32((bf16_t)(zz[d] & 0xffffu)) > 0.f)) lo = f32_to_bf16(bf16_to_f32((bf16_t)lo) * slope);
        if (!(bf16_to_f32((bf16_t)(zz[d] >> 16)) > 0.f)) hi = f32_to_bf16(bf16_to_f32((bf16_t)hi) * slope);
        gv[d] = lo | (hi << 16);
      }
      v = make_uint4(gv[0], gv[1], gv[2], gv[3]);
    }
    *reinterpret_cast<uint4*>(g + di) = v;
  } else {
    bf16_t v = dz[di];
    if (masked && !(bf16_to_f32(zm[zi]) > 0.f)) v = f32_to_bf16(bf16_to_f32(v) * slope);
    g[di] = v;
  }
}

struct K5Plan {
  int tiles_w, tiles_h, tiles_total, chunks, tiles_per_chunk;
  int bf_tiles_w, bf_tiles_h, bf_units, bf_chunks, bf_units_per_chunk;   // matrix-core backward-filter
  size_t wp_bytes, part_bytes, partdb_bytes;
};

size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

// cin / cout: channels of the input-side / output-side tensor of the layer
K5Plan k5_plan(const h3d_tensor* t, int cin, int cout, int op) {
  K5Plan p{};
  p.tiles_w = (int)cdiv(t->w, K5_TW);
  p.tiles_h = (int)cdiv(t->h, K5_TH);
  const int64_t total = (int64_t)t->n * t->d * p.tiles_w * p.tiles_h;
  p.tiles_total = (int)total;
  const int acc_c = op == H3D_OP_BWD_DATA ? cin : cout, loop_c = op == H3D_OP_BWD_DATA ? cout : cin;
  const int64_t cobs = cdiv(acc_c, K5_COB);
  const size_t alu_bytes = (size_t)cobs * loop_c * K5_TAPS * K5_COB * sizeof(float);
  const size_t mfma_bytes = (size_t)cdiv(acc_c, KM_COB) * cdiv(loop_c, KM_CIB) * K5_TAPS * KM_COB * KM_CIB * sizeof(bf16_t);
  p.wp_bytes = up256(alu_bytes > mfma_bytes ? alu_bytes : mfma_bytes);   // either form of the packed filter fits
  int64_t chunks = cdiv(1024, (int64_t)cin * cdiv(cout, K5_COB));
  if (chunks > 128) chunks = 128;
  if (chunks > total) chunks = total;
  if (chunks < 1) chunks = 1;
  p.chunks = (int)chunks;
  p.tiles_per_chunk = (int)cdiv(total, chunks);
  p.bf_tiles_w = (int)cdiv(t->w, KB_TW);
  p.bf_tiles_h = (int)cdiv(t->h, KB_TH);
  const int64_t units = (int64_t)t->n * t->d * p.bf_tiles_w * p.bf_tiles_h;
  p.bf_units = (int)units;
  int64_t bf_chunks = cdiv(1024, 5 * cdiv(cin, KB_C) * cdiv(cout, KB_C));
  if (bf_chunks > 64) bf_chunks = 64;
  if (bf_chunks > units) bf_chunks = units;
  if (bf_chunks < 1) bf_chunks = 1;
  p.bf_chunks = (int)bf_chunks;
  p.bf_units_per_chunk = (int)cdiv(units, bf_chunks);
  const int64_t most = chunks > bf_chunks ? chunks : bf_chunks;   // either form of the partial sums fits
  p.part_bytes = up256((size_t)most * cout * cin * K5_TAPS * sizeof(float));
  p.partdb_bytes = up256((size_t)most * cout * sizeof(float));
  return p;
}

// the planes a 5-wide window around the interior reaches: inside the volume they must be stored
bool k5_halo_ok(const h3d_tensor* t) {
  if (t->d == 0) return true;
  const int64_t below = t->d_offset, above = t->d_global - t->d_offset - t->d;
  return (below < 2 ? below : 2) <= t->halo_lo && (above < 2 ? above : 2) <= t->halo_hi;
}

h3d_status k5_check_pair(void* handle, const h3d_tensor* a, const h3d_tensor* b, const char* what) {
  H3D_TRY(check_tensor_packed(handle, a, what));
  H3D_TRY(check_tensor_packed(handle, b, what));
  if (!same_shard(a, b)) return fail(handle, H3D_EINVAL, "%s: the two tensors are not the same shard (n, d, h, w, offsets, dtype)", what);
  if (a->c < 1 || b->c < 1) return fail(handle, H3D_EINVAL, "%s: at least one channel on each side", what);
  if ((int64_t)a->n * cdiv(a->c > b->c ? a->c : b->c, K5_COB) > 65535 || a->d > 65535)
    return fail(handle, H3D_EUNSUPPORTED, "%s: more than 65535 planes or sample x channel blocks", what);
  if ((int64_t)a->n * a->d * cdiv(a->h, K5_TH) * cdiv(a->w, K5_TW) >= ((int64_t)1 << 31))
    return fail(handle, H3D_EUNSUPPORTED, "%s: too many tiles", what);
  return H3D_OK;
}

K5Args k5_args(const h3d_tensor* in, const h3d_tensor* out, const h3d_tensor* z, const K5Plan& p, int acc_c, float slope_in,
               float slope_out) {
  K5Args a{};
  a.in = make_geo(in);
  a.out = make_geo(out);
  a.zg = z ? make_geo(z) : a.in;
  const int64_t lo = -(int64_t)in->halo_lo > -in->d_offset ? -(int64_t)in->halo_lo : -in->d_offset;
  const int64_t hi_s = (int64_t)in->d + in->halo_hi, hi_v = in->d_global - in->d_offset;
  a.pmin = (int)lo;
  a.pmax = (int)(hi_s < hi_v ? hi_s : hi_v);
  if (z) {   // the mask tensor may store fewer planes than the gradient: both must cover what is read
    const int64_t zlo = -(int64_t)z->halo_lo, zhi = (int64_t)z->d + z->halo_hi;
    if (a.pmin < zlo) a.pmin = (int)zlo;
    if (a.pmax > zhi) a.pmax = (int)zhi;
  }
  a.tiles_w = p.tiles_w;
  a.tiles_h = p.tiles_h;
  a.cobs = (int)cdiv(acc_c, K5_COB);
  a.slope_in = slope_in;
  a.slope_out = slope_out;
  return a;
}

template <typename T>
void k5_launch_pack(const void* w, float* wp, int cin, int cout, int transposed, hipStream_t s) {
  const int loopc = transposed ? cout : cin, accc = transposed ? cin : cout;
  const int64_t total = cdiv(accc, K5_COB) * (int64_t)loopc * K5_TAPS * K5_COB;
  hipLaunchKernelGGL((k5_pack_w_kernel<T>), dim3((unsigned)cdiv(total, 256)), dim3(256), 0, s, (const T*)w, wp, cin, cout, transposed, total);
}

template <typename T>
void k5_launch_conv(const h3d_tensor* in, const h3d_tensor* z, const float* wp, const float* bias, h3d_tensor* out, const K5Args& a,
                    hipStream_t s) {
  const dim3 grid((unsigned)(a.tiles_w * a.tiles_h), (unsigned)in->d, (unsigned)(in->n * a.cobs));
  if (z)
    hipLaunchKernelGGL((k5_conv_kernel<T, true>), grid, dim3(256), 0, s, (const T*)in->data, (const T*)z->data, wp, bias, (T*)out->data, a);
  else
    hipLaunchKernelGGL((k5_conv_kernel<T, false>), grid, dim3(256), 0, s, (const T*)in->data, (const T*)nullptr, wp, bias, (T*)out->data, a);
}

template <typename T>
void k5_launch_bwf(const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* part, float* part_db, const K5Args& a,
                   const K5Plan& p, hipStream_t s) {
  const dim3 grid((unsigned)p.chunks, (unsigned)x->c, (unsigned)a.cobs);
  if (z)
    hipLaunchKernelGGL((k5_bwf_kernel<T, true>), grid, dim3(256), 0, s, (const T*)x->data, (const T*)dz->data, (const T*)z->data, part,
                       part_db, a, p.tiles_total, p.tiles_per_chunk);
  else
    hipLaunchKernelGGL((k5_bwf_kernel<T, false>), grid, dim3(256), 0, s, (const T*)x->data, (const T*)dz->data, (const T*)nullptr, part,
                       part_db, a, p.tiles_total, p.tiles_per_chunk);
}

// bf16 forward / backward-data on the matrix cores: `in` is the staged tensor, `out` the written one
void k5_launch_mfma(const h3d_tensor* in, const void* w, int cin, int cout, int transposed, const float* bias, h3d_tensor* out,
                    K5Args a, void* ws, hipStream_t s) {
  const int loopc = transposed ? cout : cin, accc = transposed ? cin : cout;
  const int cics = (int)cdiv(loopc, KM_CIB), cobs = (int)cdiv(accc, KM_COB);
  const int64_t total = (int64_t)cobs * cics * K5_TAPS * KM_COB * KM_CIB;
  bf16_t* wpk = (bf16_t*)ws;
  hipLaunchKernelGGL(k5_pack_w_mfma_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, s, (const bf16_t*)w, wpk, cin, cout, transposed,
                     cics, total);
  a.tiles_w = (int)cdiv(in->w, KM_TW);
  a.tiles_h = (int)cdiv(in->h, KM_TH);
  a.cobs = cobs;
  const dim3 grid((unsigned)(a.tiles_w * a.tiles_h), (unsigned)in->d, (unsigned)(in->n * cobs));
  hipLaunchKernelGGL(k5_mfma_kernel, grid, dim3(256), 0, s, (const bf16_t*)in->data, (const bf16_t*)wpk, bias, (bf16_t*)out->data, a, cics);
}

// g = dz * act'(z) into `g` (every stored plane of dz)
void k5_launch_grad(const h3d_tensor* dz, const h3d_tensor* z, void* g, float slope, hipStream_t s) {
  const Geo dg = make_geo(dz), zg = make_geo(z);
  const bool vec = dg.plane % 8 == 0 && (((uintptr_t)dz->data | (uintptr_t)z->data) & 15) == 0;
  const int64_t pieces = (int64_t)dz->n * dz->c * dg.ds * (dg.plane / (vec ? 8 : 1));
  if (pieces == 0) return;
  if (vec)
    hipLaunchKernelGGL((k5_grad_kernel<8>), dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, s, (const bf16_t*)dz->data,
                       (const bf16_t*)z->data, (bf16_t*)g, dg, zg, slope, pieces);
  else
    hipLaunchKernelGGL((k5_grad_kernel<1>), dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, s, (const bf16_t*)dz->data,
                       (const bf16_t*)z->data, (bf16_t*)g, dg, zg, slope, pieces);
}

bool bad_act(int act) { return act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY; }

}  // namespace
}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_conv3d_k5_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* z) {
  if (!handle || !x || !z || x->c < 1 || z->c < 1 || x->n < 0 || x->d < 0 || x->h < 0 || x->w < 0) return 0;
  const K5Plan p = k5_plan(x, x->c, z->c, op);
  switch (op) {
    case H3D_OP_FWD:
      return p.wp_bytes;
    case H3D_OP_BWD_DATA:   // bf16: room for g = dz * act'(z) on every stored plane of dz (z is the output-side descriptor here)
      return p.wp_bytes + (z->dtype == H3D_BF16 ? up256((size_t)z->n * z->c * (z->halo_lo + z->d + z->halo_hi) * z->h * z->w * sizeof(bf16_t)) : 0);
    case H3D_OP_BWD_FILTER:   // bf16: room for g as in backward-data
      return p.part_bytes + p.partdb_bytes +
             (z->dtype == H3D_BF16 ? up256((size_t)z->n * z->c * (z->halo_lo + z->d + z->halo_hi) * z->h * z->w * sizeof(bf16_t)) : 0);
    default:
      return 0;
  }
}

extern "C" h3d_status h3d_conv3d_k5_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* z, int act,
                                        float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!x || !z) return fail(handle, H3D_EINVAL, "conv3d_k5_fwd: NULL descriptor");
  H3D_TRY(k5_check_pair(handle, x, z, "conv3d_k5_fwd"));
  if (!w) return fail(handle, H3D_EINVAL, "conv3d_k5_fwd: NULL weights");
  if (bad_act(act)) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  if (!k5_halo_ok(x)) return fail(handle, H3D_EHALO, "conv3d_k5_fwd: x must store two halo planes on every side that is inside the volume");
  if (!ws || ws_bytes < h3d_conv3d_k5_workspace_bytes(handle, H3D_OP_FWD, x, z)) return fail(handle, H3D_EWORKSPACE, "conv3d_k5_fwd: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_k5_fwd: workspace must be 256-byte aligned");
  const K5Plan p = k5_plan(x, x->c, z->c, H3D_OP_FWD);
  if (p.tiles_total == 0) return H3D_OK;
  hipStream_t s = (hipStream_t)stream;
  float* wp = (float*)ws;
  const K5Args a = k5_args(x, z, nullptr, p, z->c, 1.f, act_slope(act, alpha));
  if (x->dtype == H3D_F32) { k5_launch_pack<float>(w, wp, x->c, z->c, 0, s); k5_launch_conv<float>(x, nullptr, wp, bias, z, a, s); }
  else k5_launch_mfma(x, w, x->c, z->c, 0, bias, z, a, ws, s);
  return launch_status(handle, "conv3d_k5_fwd");
}

extern "C" h3d_status h3d_conv3d_k5_bwd_data(void* handle, const h3d_tensor* dz, const h3d_tensor* z, const void* w, h3d_tensor* dx,
                                             int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!dz || !dx) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_data: NULL descriptor");
  H3D_TRY(k5_check_pair(handle, dx, dz, "conv3d_k5_bwd_data"));
  if (!w) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_data: NULL weights");
  if (bad_act(act)) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  if (act == H3D_ACT_NONE) z = nullptr;
  if (!k5_halo_ok(dz)) return fail(handle, H3D_EHALO, "conv3d_k5_bwd_data: dz must store two halo planes on every side that is inside the volume");
  if (z) {
    H3D_TRY(check_tensor_packed(handle, z, "z"));
    if (!same_shard(z, dz) || z->c != dz->c) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_data: z and dz shapes differ");
    if (!k5_halo_ok(z)) return fail(handle, H3D_EHALO, "conv3d_k5_bwd_data: z must store two halo planes on every side that is inside the volume");
  }
  if (!ws || ws_bytes < h3d_conv3d_k5_workspace_bytes(handle, H3D_OP_BWD_DATA, dx, dz)) return fail(handle, H3D_EWORKSPACE, "conv3d_k5_bwd_data: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_data: workspace must be 256-byte aligned");
  const K5Plan p = k5_plan(dx, dx->c, dz->c, H3D_OP_BWD_DATA);
  if (p.tiles_total == 0) return H3D_OK;
  hipStream_t s = (hipStream_t)stream;
  float* wp = (float*)ws;
  const K5Args a = k5_args(dz, dx, z, p, dx->c, act_slope(act, alpha), 1.f);
  if (dz->dtype == H3D_F32) { k5_launch_pack<float>(w, wp, dx->c, dz->c, 1, s); k5_launch_conv<float>(dz, z, wp, nullptr, dx, a, s); }
  else if (!z) k5_launch_mfma(dz, w, dx->c, dz->c, 1, nullptr, dx, a, ws, s);
  else {
    // the masked gradient once, then the kernel without a mask (`a` keeps the plane range that dz and z both store)
    h3d_tensor gt = *dz;
    gt.data = (char*)ws + p.wp_bytes;
    k5_launch_grad(dz, z, gt.data, a.slope_in, s);
    k5_launch_mfma(&gt, w, dx->c, dz->c, 1, nullptr, dx, a, ws, s);
  }
  return launch_status(handle, "conv3d_k5_bwd_data");
}

extern "C" h3d_status h3d_conv3d_k5_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                                               float* db, int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!x || !dz) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_filter: NULL descriptor");
  H3D_TRY(k5_check_pair(handle, x, dz, "conv3d_k5_bwd_filter"));
  if (!dw) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_filter: NULL dw");
  if (bad_act(act)) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  if (act == H3D_ACT_NONE) z = nullptr;
  if (!k5_halo_ok(x)) return fail(handle, H3D_EHALO, "conv3d_k5_bwd_filter: x must store two halo planes on every side that is inside the volume");
  if (z) {
    H3D_TRY(check_tensor_packed(handle, z, "z"));
    if (!same_shard(z, dz) || z->c != dz->c) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_filter: z and dz shapes differ");
  }
  if (!ws || ws_bytes < h3d_conv3d_k5_workspace_bytes(handle, H3D_OP_BWD_FILTER, x, dz)) return fail(handle, H3D_EWORKSPACE, "conv3d_k5_bwd_filter: workspace too small");
  if ((uintptr_t)ws & 255) return fail(handle, H3D_EINVAL, "conv3d_k5_bwd_filter: workspace must be 256-byte aligned");
  const K5Plan p = k5_plan(x, x->c, dz->c, H3D_OP_BWD_FILTER);
  hipStream_t s = (hipStream_t)stream;
  float* part = (float*)ws;
  float* part_db = (float*)((char*)ws + p.part_bytes);
  // the mask is read on the interior only: the planes of the saved output that exist do not limit x's window
  K5Args a = k5_args(x, dz, nullptr, p, dz->c, act_slope(act, alpha), 1.f);
  if (z) a.zg = make_geo(z);
  const bool aligned16 = (((uintptr_t)x->data | (uintptr_t)dz->data | (uintptr_t)(z ? z->data : nullptr)) & 15) == 0;
  int chunks = p.chunks;
  if (x->dtype == H3D_F32) {
    k5_launch_bwf<float>(x, dz, z, part, part_db, a, p, s);
  } else if (x->w % 8 == 0 && aligned16) {   // matrix cores: whole 16-byte pieces of 8 voxels
    chunks = p.bf_chunks;
    a.tiles_w = p.bf_tiles_w;
    a.tiles_h = p.bf_tiles_h;
    const int cibs = (int)cdiv(x->c, KB_C), cobs = (int)cdiv(dz->c, KB_C);
    const dim3 grid((unsigned)chunks, 5u, (unsigned)(cobs * cibs));
    const void* gsrc = dz->data;
    if (z) {   // the masked gradient once (every (kd, ci block) workgroup reads it), then the kernel without a mask
      void* gbuf = (char*)ws + p.part_bytes + p.partdb_bytes;
      k5_launch_grad(dz, z, gbuf, a.slope_in, s);
      gsrc = gbuf;
    }
    hipLaunchKernelGGL(k5_bwf_mfma_kernel, grid, dim3(KB_THREADS), 0, s, (const bf16_t*)x->data, (const bf16_t*)gsrc, part, part_db, a,
                       p.bf_units, p.bf_units_per_chunk, cibs);
  } else {
    k5_launch_bwf<bf16_t>(x, dz, z, part, part_db, a, p, s);
  }
  const int64_t nw = (int64_t)dz->c * x->c * K5_TAPS;
  hipLaunchKernelGGL(k5_reduce_kernel, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, s, (const float*)part, dw, nw, chunks);
  if (db) hipLaunchKernelGGL(k5_reduce_kernel, dim3((unsigned)cdiv(dz->c, 256)), dim3(256), 0, s, (const float*)part_db, db, (int64_t)dz->c, chunks);
  return launch_status(handle, "conv3d_k5_bwd_filter");
}
