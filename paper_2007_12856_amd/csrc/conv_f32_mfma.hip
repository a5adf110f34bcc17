// 3x3x3 convolution passes (Sec. III-C: FP, BD, BF) on fp32 tensors, on the matrix cores: v_mfma_f32_16x16x4_f32,
// fp32 products and fp32 accumulation (the paper's own precision).  The vector-ALU kernels of conv_direct.hip stay as
// the fallback for tensors these kernels' 32-bit offsets cannot address.
//
//  * forward / backward-data (one kernel; BD = the same correlation of g = dz * act'(z) with the filter transposed and
//    reversed by the pack kernel): implicit GEMM with M = 16 voxels of a row, N = 16 output channels, K = 4 input
//    channels of one tap.  A workgroup of four wavefronts owns 4 planes x 8 rows x 32 columns x (16 CB) output
//    channels, a wavefront one plane: 16 CB accumulator tiles.  Per group of 4 input channels the tile with its halo
//    (6 x 10 x 34 voxels) and the 27 x 4 x 16 CB weights are staged in LDS; per (kd, kw) the 10 input rows are read
//    once (20 fragments) and feed 3 kh x 16 CB products.  The result leaves as 16-byte stores (4 voxels of one channel
//    per lane).  Two workgroups per CU: one stages while the other multiplies.
//  * backward-filter: M = 16 input channels, N = 16 output channels, K = 4 voxels of a row.  A workgroup owns a
//    16 x 16 block of the filter and a fixed chunk of 4-row x 32-column tiles of the voxel range; each wavefront takes
//    one row of the tile and keeps 27 accumulator tiles (one per tap) plus one for the bias gradient (the product of g
//    with a column of ones).  The four wavefronts' sums are added in wavefront order, the chunks' partial sums in
//    chunk order by a second kernel: the same bits on every run.
//  * tile variants, chosen by shape alone (so a shard, a plane-run view and the whole slab sum every voxel in the same
//    order): 2-row tiles when the 8-row tiles would leave most of the chip idle; 16-column tiles for volumes at most 16
//    voxels wide; thin forms for a side with at most 4 channels (a first layer's BD and BF), where three taps share one
//    product in the rows / columns of the 16 x 16 tile that would otherwise be padding.
//  * every load goes through a buffer resource: an element outside the volume, or of a channel the tensor does not
//    have, gets an offset beyond the resource and reads as zero without a branch.
#include <algorithm>

#include "common.h"

namespace h3d {

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {
// Loads go through raw buffer resources: an element outside the volume (or of a channel the tensor does not have) gets
// the byte offset F32_OOB, which lies beyond the resource's range and reads as zero without a branch.  The channel is
// added as a scalar offset (the range check looks at the vector offset alone).
constexpr int F32_OOB = (int)0x80000000;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t f32_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                           (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
// soff = 4 * channel * channel stride: below 2^31 because a whole sample is (fits_buf on the host)
__device__ __forceinline__ float f32_load(__amdgpu_buffer_rsrc_t rs, int voff, uint32_t soff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, (int)__builtin_amdgcn_readfirstlane(soff), 0));
}
// lane i of every row of 16 lanes receives the value of lane i + N of that row (zero beyond the row's end)
template <int N>
__device__ __forceinline__ float row_shl(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + N, 0xf, 0xf, true));
}
}  // namespace

// -------------------------------------------------------------------------------------- forward / backward-data
constexpr int FT_P = 4;                            // output tile: planes; rows = the template parameter TR (8, or 2 when the
                                                   // volume has too few 8-row tiles to fill the chip); columns = 16 HV (two
                                                   // 16-voxel halves, or one for volumes at most 16 voxels wide)
constexpr int FX_P = FT_P + 2;                     // staged input planes
constexpr int FX_RP = 36;                          // row pitch in LDS (floats)
// channel pitch in LDS: 16 mod 64, so the four channels of a fragment read land in four different bank groups
constexpr int fx_cs(int tr) { return (FX_P * (tr + 2) * FX_RP + 63) / 64 * 64 + 16; }

// w: [cout][cin][27] fp32 -> wk: [co group][ci group][27][4][NC]  (NC = 16 CB output channels, zeros where padded)
// fwd:      kernel-view (co_k, ci_k, t) = w[co_k][ci_k][t]
// bwd-data: kernel-view (co_k, ci_k, t) = w[ci_k][co_k][26 - t]      (cin_k = cout, cout_k = cin)
__global__ void pack_w_f32_mfma_kernel(const float* __restrict__ w, float* __restrict__ wk, int cin, int cout, int transpose,
                                       int ncig, int nc, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cin_k = transpose ? cout : cin, cout_k = transpose ? cin : cout;
  const int j = (int)(i % nc);
  const int c = (int)((i / nc) % 4);
  const int t = (int)((i / (4 * nc)) % 27);
  const int cig = (int)((i / (108 * (int64_t)nc)) % ncig);
  const int cog = (int)(i / (108 * (int64_t)nc * ncig));
  const int ok = cog * nc + j, ik = cig * 4 + c;
  float v = 0.f;
  if (ok < cout_k && ik < cin_k) v = transpose ? w[((int64_t)ik * cin + ok) * 27 + (26 - t)] : w[((int64_t)ok * cin + ik) * 27 + t];
  wk[i] = v;
}

// Thin output side (at most 4 output channels: the BD of a first layer): the 16 columns of a product hold (kh, co) =
// column 4 kh + co, so one product covers the three kh taps.  wk: [ci group][kd * 3 + kw][4][16], zeros where padded.
__global__ void pack_w_f32_thin_kernel(const float* __restrict__ w, float* __restrict__ wk, int cin, int cout, int transpose,
                                       int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cin_k = transpose ? cout : cin, cout_k = transpose ? cin : cout;
  const int j = (int)(i % 16);
  const int c = (int)((i / 16) % 4);
  const int dk = (int)((i / 64) % 9);
  const int cig = (int)(i / 576);
  const int kh = j / 4, ok = j % 4, ik = cig * 4 + c;
  const int t = (dk / 3) * 9 + kh * 3 + dk % 3;
  float v = 0.f;
  if (kh < 3 && ok < cout_k && ik < cin_k) v = transpose ? w[((int64_t)ik * cin + ok) * 27 + (26 - t)] : w[((int64_t)ok * cin + ik) * 27 + t];
  wk[i] = v;
}

struct F32Args {
  Geo in, mask, out;
  int cin, cout, ncig;
  int npg, nhg, nwg;      // plane groups (over the stored planes of out), row groups, column groups
  float out_slope, mask_slope;
  int vec;                // 16-byte stores allowed
};

template <int CB, int TR, int HV, bool MASKED, bool THIN = false>
__global__ void __launch_bounds__(256, 2) conv3d_f32_mfma_kernel(const float* __restrict__ in, const float* __restrict__ mask,
                                                                 const float* __restrict__ wk, const float* __restrict__ bias,
                                                                 float* __restrict__ out, F32Args a) {
  static_assert(!THIN || CB == 1, "the thin form has one block of columns");
  constexpr int NC = 16 * CB;
  constexpr int WSZ = (THIN ? 9 : 27) * 4 * NC;    // weights of one channel group (floats)
  constexpr int FT_R = TR, FX_R = TR + 2;          // output rows, staged input rows
  constexpr int FT_W = 16 * HV, FX_C = FT_W + 2;   // output columns, staged input columns
  constexpr int FX_PS = FX_R * FX_RP;              // plane pitch
  constexpr int FX_CS = fx_cs(TR);                 // channel pitch
  constexpr int FX_SP = FX_P * FX_R * FX_C;        // staged voxels per channel (2040 for 8 rows)
  constexpr int FX_PT = (FX_SP + 255) / 256;       // per thread and channel (8)
  __shared__ float lds_x[4 * FX_CS];
  __shared__ __attribute__((aligned(16))) float lds_w[WSZ];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int W = a.out.w, H = a.out.h;
  int t = blockIdx.x;
  const int wg = t % a.nwg; t /= a.nwg;
  const int hg = t % a.nhg; t /= a.nhg;
  const int pg = t % a.npg;
  const int n = t / a.npg;
  const int cog = blockIdx.y;
  const int ps0 = pg * FT_P, h0 = hg * FT_R, w0 = wg * FT_W;

  // what this thread stages of every channel: byte offsets in the channel (F32_OOB: outside the volume, reads as zero)
  // and offsets in LDS
  int xoff[FX_PT], moff[FX_PT], loff[FX_PT];
#pragma unroll
  for (int i = 0; i < FX_PT; ++i) {
    const int s = tid + 256 * i;
    const int col = s % FX_C, row = (s / FX_C) % FX_R, pl = s / (FX_C * FX_R);
    loff[i] = s < FX_SP ? pl * FX_PS + row * FX_RP + col : -1;
    const int q = ps0 - a.out.hlo - 1 + pl;                 // local plane index of the input
    const int64_t gq = a.in.doff + q;
    const int sp = q + a.in.hlo, hh = h0 - 1 + row, ww = w0 - 1 + col;
    const bool ok = s < FX_SP && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && hh >= 0 && hh < H && ww >= 0 && ww < W;
    xoff[i] = ok ? 4 * (int)(sp * a.in.plane + (int64_t)hh * W + ww) : F32_OOB;
    if (MASKED) {
      const int sm = q + a.mask.hlo;
      const bool mok = ok && sm >= 0 && sm < a.mask.ds;
      moff[i] = mok ? 4 * (int)(sm * a.mask.plane + (int64_t)hh * W + ww) : F32_OOB;
      if (!mok) xoff[i] = F32_OOB;
    }
  }

  const int ps = ps0 + wave;                               // stored plane of out this wavefront computes
  const bool live = ps < a.out.ds;
  const int64_t gp = a.out.doff + ps - a.out.hlo;
  const bool inside = gp >= 0 && gp < a.out.dglob;

  // accumulators: one per output row, starting from the bias — or, in the thin form, one per INPUT row (its three kh
  // contributions sit in columns 4 kh + co and meet the output rows they belong to in the epilogue)
  constexpr int NAR = THIN ? FX_R : FT_R;
  f32x4 acc[CB][NAR][HV];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int co = cog * NC + cb * 16 + (lane & 15);
    const float b = (!THIN && bias && co < a.cout) ? bias[co] : 0.f;
#pragma unroll
    for (int r = 0; r < NAR; ++r)
#pragma unroll
      for (int hf = 0; hf < HV; ++hf) acc[cb][r][hf] = f32x4{b, b, b, b};
  }

  const float* xw = lds_x + (lane >> 4) * FX_CS + wave * FX_PS + (lane & 15);
  const float* ww_ = lds_w + (lane >> 4) * NC + (lane & 15);
  const __amdgpu_buffer_rsrc_t rs_in = f32_rsrc(in + (int64_t)n * a.in.nstride, (uint32_t)(a.in.nstride * 4));
  const __amdgpu_buffer_rsrc_t rs_mk = f32_rsrc(MASKED ? mask + (int64_t)n * a.mask.nstride : in, (uint32_t)(a.mask.nstride * 4));

  for (int cig = 0; cig < a.ncig; ++cig) {
    // ---- stage 4 input channels (tile + halo) and their weights
    float v[4][FX_PT];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int ci = cig * 4 + c;
      const bool cok = ci < a.cin;                  // uniform
      const uint32_t xs = 4u * ci * (uint32_t)a.in.cstride, ms = MASKED ? 4u * ci * (uint32_t)a.mask.cstride : 0u;
#pragma unroll
      for (int i = 0; i < FX_PT; ++i) {
        float x = f32_load(rs_in, cok ? xoff[i] : F32_OOB, xs);
        if (MASKED) {
          const float m = f32_load(rs_mk, cok ? moff[i] : F32_OOB, ms);
          x = m > 0.f ? x : x * a.mask_slope;
        }
        v[c][i] = x;
      }
    }
    const f32x4* wsrc = reinterpret_cast<const f32x4*>(wk + ((int64_t)cog * a.ncig + cig) * WSZ);   // (thin: one column group)
    f32x4 wv[(WSZ / 4 + 255) / 256];
#pragma unroll
    for (int i = 0; i < (WSZ / 4 + 255) / 256; ++i) {
      const int j = tid + 256 * i;
      wv[i] = j < WSZ / 4 ? wsrc[j] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();                                       // everyone is done with the previous group's tile
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int i = 0; i < FX_PT; ++i)
        if (loff[i] >= 0) lds_x[c * FX_CS + loff[i]] = v[c][i];
#pragma unroll
    for (int i = 0; i < (WSZ / 4 + 255) / 256; ++i) {
      const int j = tid + 256 * i;
      if (j < WSZ / 4) reinterpret_cast<f32x4*>(lds_w)[j] = wv[i];
    }
    __syncthreads();

    // ---- products: per (kd, kw) the ten rows are read once and meet the three kh weight fragments
    if (live) {
#pragma unroll
      for (int kd = 0; kd < 3; ++kd) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          float bx[FX_R][HV];
#pragma unroll
          for (int r = 0; r < FX_R; ++r)
#pragma unroll
            for (int hf = 0; hf < HV; ++hf) bx[r][hf] = xw[kd * FX_PS + r * FX_RP + hf * 16 + kw];
          if (THIN) {
            const float aw = ww_[(kd * 3 + kw) * 4 * NC];
#pragma unroll
            for (int r = 0; r < FX_R; ++r)
#pragma unroll
              for (int hf = 0; hf < HV; ++hf)
                acc[0][r][hf] = __builtin_amdgcn_mfma_f32_16x16x4f32(bx[r][hf], aw, acc[0][r][hf], 0, 0, 0);
          } else {
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
#pragma unroll
              for (int cb = 0; cb < CB; ++cb) {
                const float aw = ww_[((kd * 3 + kh) * 3 + kw) * 4 * NC + cb * 16];
#pragma unroll
                for (int r = 0; r < FT_R; ++r)
#pragma unroll
                  for (int hf = 0; hf < HV; ++hf)
                    acc[cb][r][hf] = __builtin_amdgcn_mfma_f32_16x16x4f32(bx[r + kh][hf], aw, acc[cb][r][hf], 0, 0, 0);
              }
            }
          }
        }
      }
    }
  }

  // ---- epilogue: activation, zero outside the volume, 16-byte stores of 4 voxels of one channel
  if (!live) return;
  float* on = out + (int64_t)n * a.out.nstride + (int64_t)ps * a.out.plane;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int co = cog * NC + cb * 16 + (lane & 15);
    const bool co_ok = co < a.cout;       // (tested at the store: the lane exchange of the thin form needs whole rows of lanes)
    float* oc = on + (int64_t)co * a.out.cstride;
#pragma unroll
    for (int r = 0; r < FT_R; ++r) {
      const int h = h0 + r;
      if (h >= H) continue;
#pragma unroll
      for (int hf = 0; hf < HV; ++hf) {
        const int wc = w0 + hf * 16 + 4 * (lane >> 4);
        if (wc >= W) continue;
        f32x4 o;
        if (THIN) {
          // output row r = input rows r, r + 1, r + 2 under kh = 0, 1, 2: columns co, 4 + co, 8 + co
          const float b = (bias && co < a.cout) ? bias[co] : 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            o[j] = ((acc[0][r][hf][j] + row_shl<4>(acc[0][r + 1][hf][j])) + row_shl<8>(acc[0][r + 2][hf][j])) + b;
        } else {
          o = acc[cb][r][hf];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float x = o[j];
          if (!(x > 0.f)) x *= a.out_slope;
          o[j] = inside ? x : 0.f;
        }
        float* p = oc + (int64_t)h * W + wc;
        if (!co_ok) continue;
        if (a.vec && wc + 3 < W) {
          *reinterpret_cast<f32x4*>(p) = o;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (wc + j < W) p[j] = o[j];
        }
      }
    }
  }
}

static int f32_cb(int cout_k) { return cout_k <= 16 ? 1 : 2; }

// a whole sample (all channels, with the tensor's real strides) within 2^31 bytes: what a buffer resource and the
// 32-bit byte offsets of the kernels can address
static bool fits_buf(const h3d_tensor* t) { return sample_span(t) < ((int64_t)1 << 29); }

bool f32_mfma_fwd_supported(const h3d_tensor* in, const h3d_tensor* out) {
  return in->dtype == H3D_F32 && out->dtype == H3D_F32 && in->c > 0 && out->c > 0 && fits_buf(in) && fits_buf(out);
}

size_t f32_mfma_fwd_ws_bytes(int cin_k, int cout_k) {
  const int nc = 16 * f32_cb(cout_k);
  return (size_t)cdiv(cout_k, nc) * cdiv(cin_k, 4) * 108 * nc * sizeof(float);
}

h3d_status conv3d_f32_mfma(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                           h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                           hipStream_t stream) {
  const int cin_k = in->c, cout_k = out->c;
  const int cin = transpose ? cout_k : cin_k, cout = transpose ? cin_k : cout_k;
  const bool thin = cout_k <= 4;
  const int cb = f32_cb(cout_k), nc = 16 * cb;
  if (!ws || ws_bytes < f32_mfma_fwd_ws_bytes(cin_k, cout_k)) return fail(handle, H3D_EWORKSPACE, "conv3d: workspace too small");
  if (mask && !fits_buf(mask)) return fail(handle, H3D_EUNSUPPORTED, "conv3d: z too large for this kernel");
  F32Args a;
  a.in = make_geo(in);
  a.mask = mask ? make_geo(mask) : a.in;
  a.out = make_geo(out);
  a.cin = cin_k; a.cout = cout_k; a.ncig = (int)cdiv(cin_k, 4);
  const int hv = out->w <= 16 ? 1 : 2;
  a.npg = (int)cdiv(a.out.ds, FT_P); a.nwg = (int)cdiv(out->w, 16 * hv);
  const int ncog = (int)cdiv(cout_k, nc);
  // 8-row tiles unless they would leave most of the chip idle: then 2-row tiles, four times as many workgroups
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  const int tr = ((int64_t)out->n * a.npg * cdiv(out->h, 8) * a.nwg * ncog < 2 * (int64_t)num_cu && out->h > 2) ? 2 : 8;
  a.nhg = (int)cdiv(out->h, tr);
  a.out_slope = out_slope; a.mask_slope = mask_slope;
  a.vec = (out->w % 4 == 0) && (a.out.cstride % 4 == 0) && (a.out.nstride % 4 == 0) && ((uintptr_t)out->data % 16 == 0);
  const int64_t tiles = (int64_t)out->n * a.npg * a.nhg * a.nwg;
  if (tiles == 0) return H3D_OK;
  if (tiles >= ((int64_t)1 << 31) || ncog > 65535) return fail(handle, H3D_EINVAL, "conv3d: too many blocks");
  const int64_t nw = thin ? (int64_t)a.ncig * 576 : (int64_t)ncog * a.ncig * 108 * nc;
  if (thin)
    hipLaunchKernelGGL(pack_w_f32_thin_kernel, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, stream, (const float*)w, (float*)ws,
                       cin, cout, transpose ? 1 : 0, nw);
  else
    hipLaunchKernelGGL(pack_w_f32_mfma_kernel, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, stream, (const float*)w, (float*)ws,
                       cin, cout, transpose ? 1 : 0, a.ncig, nc, nw);
  const dim3 g((unsigned)tiles, (unsigned)ncog);
#define H3D_F32_LAUNCH(CBV, TRV, HVV, MK, TH)                                                                           \
  hipLaunchKernelGGL((conv3d_f32_mfma_kernel<CBV, TRV, HVV, MK, TH>), g, dim3(256), 0, stream, (const float*)in->data,  \
                     (const float*)(mask ? mask->data : nullptr), (const float*)ws, bias, (float*)out->data, a)
#define H3D_F32_LAUNCH_M(CBV, TRV, HVV, TH)                                                                             \
  do {                                                                                                                  \
    if (mask) H3D_F32_LAUNCH(CBV, TRV, HVV, true, TH); else H3D_F32_LAUNCH(CBV, TRV, HVV, false, TH);                   \
  } while (0)
#define H3D_F32_LAUNCH_T(CBV, TH)                                                                                       \
  do {                                                                                                                  \
    if (tr == 8 && hv == 2) H3D_F32_LAUNCH_M(CBV, 8, 2, TH);                                                            \
    else if (tr == 8) H3D_F32_LAUNCH_M(CBV, 8, 1, TH);                                                                  \
    else if (hv == 2) H3D_F32_LAUNCH_M(CBV, 2, 2, TH);                                                                  \
    else H3D_F32_LAUNCH_M(CBV, 2, 1, TH);                                                                               \
  } while (0)
  if (thin) H3D_F32_LAUNCH_T(1, true);
  else if (cb == 1) H3D_F32_LAUNCH_T(1, false);
  else H3D_F32_LAUNCH_T(2, false);
#undef H3D_F32_LAUNCH_T
#undef H3D_F32_LAUNCH_M
#undef H3D_F32_LAUNCH
  if (thin) note_kernel(handle, "conv3d_f32_mfma_kernel<thin,%d,%d>", tr, hv);
  else note_kernel(handle, "conv3d_f32_mfma_kernel<%d,%d,%d>", cb, tr, hv);
  return launch_status(handle, "conv3d_f32_mfma");
}

// ------------------------------------------------------------------------------------------------ backward-filter
// tile of output voxels (one plane, 128 voxels): 4 rows x 32 columns, one row per wavefront — or, for volumes at most 16
// voxels wide (NARROW), 8 rows x 16 columns, two rows per wavefront
struct BfTile {
  int rows, cols, xr, xc, sp, rw, kc;   // tile rows / columns, staged rows / columns of x, staged voxels per channel,
};                                      // rows per wavefront, K-steps per row
constexpr BfTile bf_tile(bool narrow) {
  return narrow ? BfTile{8, 16, 10, 18, 3 * 10 * 18, 2, 4} : BfTile{4, 32, 6, 34, 3 * 6 * 34, 1, 8};
}
constexpr int BX_CS = 644;                         // channel pitch of x in LDS (>= 612 staged voxels): 4 mod 64 (a fragment
                                                   // read takes lane (c, k) to bank 4 c + k)
constexpr int BG_CS = 128 + 4;                     // channel pitch of g: 132 = 4 mod 64

struct F32BfArgs {
  Geo x, dz, z;
  int cin, cout;
  int nhg, nwg;
  int64_t tiles;            // n * d * nhg * nwg
  int tiles_per_chunk;
  float mask_slope;
};

// partial sums: [chunk][cout][cin][28] (slot 27 = bias gradient, written for ci == 0 only)
template <bool MASKED, bool NARROW>
__global__ void __launch_bounds__(256, 2) bwd_filter_f32_mfma_kernel(const float* __restrict__ x, const float* __restrict__ dz,
                                                                     const float* __restrict__ z, float* __restrict__ part,
                                                                     F32BfArgs a) {
  __shared__ float lds_x[16 * BX_CS];
  __shared__ float lds_g[16 * BG_CS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, cog = blockIdx.y, cig = blockIdx.z;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  f32x4 acc[28];
#pragma unroll
  for (int t = 0; t < 28; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  constexpr BfTile T = bf_tile(NARROW);
  constexpr int BT_R = T.rows, BT_W = T.cols, BX_R = T.xr, BX_C = T.xc, BX_SP = T.sp;
  const float* xr = lds_x + (lane & 15) * BX_CS + wave * T.rw * BX_C + (lane >> 4);
  const float* gr = lds_g + (lane & 15) * BG_CS + wave * T.rw * BT_W + (lane >> 4);

  // what this thread stages of a tile: three voxels of the x window in each of the 16 input channels, and one voxel of
  // the g tile in 8 of the 16 output channels.  The loads of the next tile are issued before the products of the present
  // one and land in registers meanwhile.
  constexpr int BX_PT = (BX_SP + 255) / 256;              // 3
  float xv[BX_PT][16], gv[8], zv[8];
  const int gs = tid & 127, gc0 = (tid >> 7) * 8;         // g: voxel of the tile, first of this thread's channels
  const int nci = min(16, a.cin - cig * 16), nco = min(16, a.cout - cog * 16);
  auto load_tile = [&](int64_t tile) {
    int64_t r = tile;
    const int wg = (int)(r % a.nwg); r /= a.nwg;
    const int hg = (int)(r % a.nhg); r /= a.nhg;
    const int p = (int)(r % D);
    const int n = (int)(r / D);
    const int h0 = hg * BT_R, w0 = wg * BT_W;
    const __amdgpu_buffer_rsrc_t rs_x = f32_rsrc(x + (int64_t)n * a.x.nstride, (uint32_t)(a.x.nstride * 4));
    const __amdgpu_buffer_rsrc_t rs_g = f32_rsrc(dz + (int64_t)n * a.dz.nstride, (uint32_t)(a.dz.nstride * 4));
    const __amdgpu_buffer_rsrc_t rs_z = f32_rsrc(MASKED ? z + (int64_t)n * a.z.nstride : dz, (uint32_t)(a.z.nstride * 4));
#pragma unroll
    for (int i = 0; i < BX_PT; ++i) {
      const int s = tid + 256 * i;
      const int col = s % BX_C, row = (s / BX_C) % BX_R, pl = s / (BX_C * BX_R);
      const int q = p + pl - 1;
      const int64_t gq = a.x.doff + q;
      const int sp = q + a.x.hlo, hh = h0 - 1 + row, ww = w0 - 1 + col;
      const bool ok = s < BX_SP && gq >= 0 && gq < a.x.dglob && sp >= 0 && sp < a.x.ds && hh >= 0 && hh < H && ww >= 0 && ww < W;
      const int vo = ok ? 4 * (int)((int64_t)sp * a.x.plane + (int64_t)hh * W + ww) : F32_OOB;
#pragma unroll
      for (int c = 0; c < 16; ++c) xv[i][c] = f32_load(rs_x, c < nci ? vo : F32_OOB, 4u * (cig * 16 + c) * (uint32_t)a.x.cstride);
    }
    const int hh = h0 + gs / BT_W, ww = w0 + gs % BT_W;
    const bool gok = hh < H && ww < W;
    const int go = gok ? 4 * (int)((int64_t)(p + a.dz.hlo) * a.dz.plane + (int64_t)hh * W + ww) : F32_OOB;
    const int zo = (MASKED && gok) ? 4 * (int)((int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)hh * W + ww) : F32_OOB;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool ok = gc0 + j < nco;                      // (gc0 differs between the two halves of the workgroup)
      gv[j] = f32_load(rs_g, ok ? go : F32_OOB, 4u * (cog * 16 + gc0 + j) * (uint32_t)a.dz.cstride);
      if (MASKED) zv[j] = f32_load(rs_z, ok ? zo : F32_OOB, 4u * (cog * 16 + gc0 + j) * (uint32_t)a.z.cstride);   // 0 where g is 0
    }
  };

  const int64_t t0 = (int64_t)chunk * a.tiles_per_chunk;
  const int64_t t1 = min(t0 + a.tiles_per_chunk, a.tiles);
  if (t0 < t1) load_tile(t0);
  for (int64_t tile = t0; tile < t1; ++tile) {
    __syncthreads();                                      // the previous tile's fragments have been read
#pragma unroll
    for (int i = 0; i < BX_PT; ++i) {
      const int s = tid + 256 * i;
      if (s < BX_SP) {
#pragma unroll
        for (int c = 0; c < 16; ++c) lds_x[c * BX_CS + s] = xv[i][c];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float v = gv[j];
      if (MASKED && !(zv[j] > 0.f)) v *= a.mask_slope;    // g = dz * act'(z)
      lds_g[(gc0 + j) * BG_CS + gs] = v;
    }
    __syncthreads();
    if (tile + 1 < t1) load_tile(tile + 1);
    // ---- this wavefront's row(s): 8 steps of 4 voxels, 27 taps + the bias gradient
#pragma unroll
    for (int rr = 0; rr < T.rw; ++rr) {
#pragma unroll 2
      for (int kc = 0; kc < T.kc; ++kc) {
        const float g = gr[rr * BT_W + 4 * kc];
        float xf[27];
#pragma unroll
        for (int t = 0; t < 27; ++t) xf[t] = xr[(t / 9) * (BX_R * BX_C) + ((t / 3) % 3 + rr) * BX_C + 4 * kc + t % 3];
#pragma unroll
        for (int t = 0; t < 27; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(xf[t], g, acc[t], 0, 0, 0);
        acc[27] = __builtin_amdgcn_mfma_f32_16x16x4f32(1.f, g, acc[27], 0, 0, 0);
        // LDS reads several products ahead of their use: six reads first, then one read per two products
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
        for (int t = 0; t < 14; ++t) {
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    }
  }

  // ---- the four wavefronts' sums, added in wavefront order through LDS (the x tile's space: 28 x 1024 B x 4 <= 41 KB)
  float* red = lds_x;
  for (int wv = 0; wv < 4; ++wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int t = 0; t < 28; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int idx = (t * 4 + j) * 64 + lane;
          if (wv == 0) red[idx] = acc[t][j];
          else if (wv < 3) red[idx] += acc[t][j];
          else acc[t][j] += red[idx];
        }
    }
  }
  if (wave != 3) return;
  // lane holds ci = 4 (lane / 16) + j, co = lane % 16 of every tap
  const int co = cog * 16 + (lane & 15);
  if (co >= a.cout) return;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int ci = cig * 16 + 4 * (lane >> 4) + j;
    if (ci >= a.cin) continue;
    float* pp = part + (((int64_t)chunk * a.cout + co) * a.cin + ci) * 28;
#pragma unroll
    for (int t = 0; t < 27; ++t) pp[t] = acc[t][j];
    if (ci == 0) pp[27] = acc[27][j];
  }
}

// Thin input side (at most 4 input channels: the BF of a first layer).  The 16 rows of a product hold (kw, ci) = row
// 4 kw + ci (kw = 3 is padding), so one product covers the three kw taps of a (kd, kh): 9 products + the bias gradient
// per K-step instead of 28, and only 4 channels of x are staged.  Little per workgroup (≤ 128 registers, 19 KB of LDS):
// four workgroups per CU.  Same partial-sum layout and reduction as the general form.
template <bool MASKED, bool NARROW>
__global__ void __launch_bounds__(256, 4) bwd_filter_f32_thin_kernel(const float* __restrict__ x, const float* __restrict__ dz,
                                                                     const float* __restrict__ z, float* __restrict__ part,
                                                                     F32BfArgs a) {
  __shared__ float lds_x[4 * BX_CS];                      // (the padding rows read at most 3 floats past a tap: inside the array)
  __shared__ float lds_g[16 * BG_CS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, cog = blockIdx.y;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  f32x4 acc[10];
#pragma unroll
  for (int t = 0; t < 10; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // A operand: lane l supplies row l % 16 = (kw, ci) at voxel l / 16 of the K-step
  constexpr BfTile T = bf_tile(NARROW);
  constexpr int BT_R = T.rows, BT_W = T.cols, BX_R = T.xr, BX_C = T.xc, BX_SP = T.sp;
  const float* xr = lds_x + (lane & 3) * BX_CS + wave * T.rw * BX_C + (lane >> 4) + ((lane & 15) >> 2);
  const float* gr = lds_g + (lane & 15) * BG_CS + wave * T.rw * BT_W + (lane >> 4);

  constexpr int BX_PT = (BX_SP + 255) / 256;              // 3
  float xv[BX_PT][4], gv[8], zv[8];
  const int gs = tid & 127, gc0 = (tid >> 7) * 8;
  const int nco = min(16, a.cout - cog * 16);
  auto load_tile = [&](int64_t tile) {
    int64_t r = tile;
    const int wg = (int)(r % a.nwg); r /= a.nwg;
    const int hg = (int)(r % a.nhg); r /= a.nhg;
    const int p = (int)(r % D);
    const int n = (int)(r / D);
    const int h0 = hg * BT_R, w0 = wg * BT_W;
    const __amdgpu_buffer_rsrc_t rs_x = f32_rsrc(x + (int64_t)n * a.x.nstride, (uint32_t)(a.x.nstride * 4));
    const __amdgpu_buffer_rsrc_t rs_g = f32_rsrc(dz + (int64_t)n * a.dz.nstride, (uint32_t)(a.dz.nstride * 4));
    const __amdgpu_buffer_rsrc_t rs_z = f32_rsrc(MASKED ? z + (int64_t)n * a.z.nstride : dz, (uint32_t)(a.z.nstride * 4));
#pragma unroll
    for (int i = 0; i < BX_PT; ++i) {
      const int s = tid + 256 * i;
      const int col = s % BX_C, row = (s / BX_C) % BX_R, pl = s / (BX_C * BX_R);
      const int q = p + pl - 1;
      const int64_t gq = a.x.doff + q;
      const int sp = q + a.x.hlo, hh = h0 - 1 + row, ww = w0 - 1 + col;
      const bool ok = s < BX_SP && gq >= 0 && gq < a.x.dglob && sp >= 0 && sp < a.x.ds && hh >= 0 && hh < H && ww >= 0 && ww < W;
      const int vo = ok ? 4 * (int)((int64_t)sp * a.x.plane + (int64_t)hh * W + ww) : F32_OOB;
#pragma unroll
      for (int c = 0; c < 4; ++c) xv[i][c] = f32_load(rs_x, c < a.cin ? vo : F32_OOB, 4u * c * (uint32_t)a.x.cstride);
    }
    const int hh = h0 + gs / BT_W, ww = w0 + gs % BT_W;
    const bool gok = hh < H && ww < W;
    const int go = gok ? 4 * (int)((int64_t)(p + a.dz.hlo) * a.dz.plane + (int64_t)hh * W + ww) : F32_OOB;
    const int zo = (MASKED && gok) ? 4 * (int)((int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)hh * W + ww) : F32_OOB;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool ok = gc0 + j < nco;
      gv[j] = f32_load(rs_g, ok ? go : F32_OOB, 4u * (cog * 16 + gc0 + j) * (uint32_t)a.dz.cstride);
      if (MASKED) zv[j] = f32_load(rs_z, ok ? zo : F32_OOB, 4u * (cog * 16 + gc0 + j) * (uint32_t)a.z.cstride);
    }
  };

  const int64_t t0 = (int64_t)chunk * a.tiles_per_chunk;
  const int64_t t1 = min(t0 + a.tiles_per_chunk, a.tiles);
  if (t0 < t1) load_tile(t0);
  for (int64_t tile = t0; tile < t1; ++tile) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < BX_PT; ++i) {
      const int s = tid + 256 * i;
      if (s < BX_SP) {
#pragma unroll
        for (int c = 0; c < 4; ++c) lds_x[c * BX_CS + s] = xv[i][c];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float v = gv[j];
      if (MASKED && !(zv[j] > 0.f)) v *= a.mask_slope;
      lds_g[(gc0 + j) * BG_CS + gs] = v;
    }
    __syncthreads();
    if (tile + 1 < t1) load_tile(tile + 1);
#pragma unroll
    for (int rr = 0; rr < T.rw; ++rr) {
#pragma unroll 2
      for (int kc = 0; kc < T.kc; ++kc) {
        const float g = gr[rr * BT_W + 4 * kc];
        float xf[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) xf[t] = xr[(t / 3) * (BX_R * BX_C) + (t % 3 + rr) * BX_C + 4 * kc];
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(xf[t], g, acc[t], 0, 0, 0);
        acc[9] = __builtin_amdgcn_mfma_f32_16x16x4f32(1.f, g, acc[9], 0, 0, 0);
      }
    }
  }

  // ---- the four wavefronts' sums in wavefront order (10 x 1 KB through the x tile's space)
  float* red = lds_x;
  for (int wv = 0; wv < 4; ++wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int t = 0; t < 10; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int idx = (t * 4 + j) * 64 + lane;
          if (wv == 0) red[idx] = acc[t][j];
          else if (wv < 3) red[idx] += acc[t][j];
          else acc[t][j] += red[idx];
        }
    }
  }
  if (wave != 3) return;
  // lane holds kw = lane / 16 (3: padding), ci = j, co = lane % 16 of every (kd, kh)
  const int co = cog * 16 + (lane & 15), kw = lane >> 4;
  if (co >= a.cout || kw >= 3) return;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j >= a.cin) continue;
    float* pp = part + (((int64_t)chunk * a.cout + co) * a.cin + j) * 28;
#pragma unroll
    for (int t = 0; t < 9; ++t) pp[t * 3 + kw] = acc[t][j];
    if (j == 0 && kw == 0) pp[27] = acc[9][0];
  }
}

// dw / db = the chunks' partial sums added in a fixed order: a block takes 16 consecutive elements of a chunk row; each
// of its 16 thread groups adds every 16th chunk in increasing order (eight loads in flight), then the 16 group sums are
// added in group order.
__global__ void __launch_bounds__(256) bwd_filter_f32_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                    float* __restrict__ db, int cin, int cout, int nchunks) {
  constexpr int G = 16;
  __shared__ float red[G][17];
  const int o = threadIdx.x & 15, cg = threadIdx.x >> 4;
  const int64_t i = (int64_t)blockIdx.x * 16 + o;
  const int64_t total = (int64_t)cout * cin * 28;
  const int t = (int)(i % 28);
  const int ci = (int)((i / 28) % cin);
  const int co = (int)(i / (28 * (int64_t)cin));
  const bool want = i < total && (t < 27 || (ci == 0 && db));
  float s = 0.f;
  if (want) {
    const float* base = part + i;
    int c = cg;
    for (; c + 7 * G < nchunks; c += 8 * G) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = base[(int64_t)(c + u * G) * total];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nchunks; c += G) s += base[(int64_t)c * total];
  }
  red[cg][o] = s;
  __syncthreads();
  if (cg == 0 && want) {
    float r = red[0][o];
#pragma unroll
    for (int k = 1; k < G; ++k) r += red[k][o];
    if (t < 27) dw[((int64_t)co * cin + ci) * 27 + t] = r;
    else db[co] = r;
  }
}

static void f32_bf_plan(const h3d_tensor* x, int cout, int64_t* tiles, int* tpc, int* nchunks) {
  const BfTile T = bf_tile(x->w <= 16);
  *tiles = (int64_t)x->n * x->d * cdiv(x->h, T.rows) * cdiv(x->w, T.cols);
  const int64_t blocks = cdiv(cout, 16) * cdiv(x->c, 16);
  const int64_t per_chunk = (int64_t)cout * x->c * 28 * 4;
  int64_t want = std::max<int64_t>(1, cdiv(1024, std::max<int64_t>(blocks, 1)));
  want = std::min<int64_t>(want, std::max<int64_t>(1, ((int64_t)64 << 20) / std::max<int64_t>(per_chunk, 1)));
  want = std::min<int64_t>(want, std::max<int64_t>(*tiles, 1));
  *tpc = (int)std::max<int64_t>(1, cdiv(*tiles, want));
  *nchunks = (int)std::max<int64_t>(1, cdiv(*tiles, *tpc));
}

bool f32_mfma_bf_supported(const h3d_tensor* x, const h3d_tensor* dz) {
  return x->dtype == H3D_F32 && dz->dtype == H3D_F32 && x->c > 0 && dz->c > 0 && cdiv(x->c, 16) <= 65535 && cdiv(dz->c, 16) <= 65535 && fits_buf(x) && fits_buf(dz);
}

size_t f32_mfma_bf_ws_bytes(const h3d_tensor* x, int cout) {
  int64_t tiles;
  int tpc, nchunks;
  f32_bf_plan(x, cout, &tiles, &tpc, &nchunks);
  return (size_t)nchunks * cout * x->c * 28 * sizeof(float);
}

h3d_status bwd_filter_f32_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                               float* db, float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  F32BfArgs a;
  a.x = make_geo(x); a.dz = make_geo(dz); a.z = z ? make_geo(z) : a.dz;
  a.cin = x->c; a.cout = dz->c; a.mask_slope = mask_slope;
  const bool narrow = x->w <= 16;
  const BfTile T = bf_tile(narrow);
  a.nhg = (int)cdiv(x->h, T.rows); a.nwg = (int)cdiv(x->w, T.cols);
  int nchunks;
  f32_bf_plan(x, a.cout, &a.tiles, &a.tiles_per_chunk, &nchunks);
  if (!ws || ws_bytes < f32_mfma_bf_ws_bytes(x, a.cout)) return fail(handle, H3D_EWORKSPACE, "conv3d_bwd_filter: workspace too small");
  if (z && !fits_buf(z)) return fail(handle, H3D_EUNSUPPORTED, "conv3d_bwd_filter: z too large for this kernel");
  const dim3 g((unsigned)nchunks, (unsigned)cdiv(a.cout, 16), (unsigned)cdiv(a.cin, 16));
  const bool thin = a.cin <= 4;
#define H3D_F32_BF(KERN, MK, NW)                                                                                        \
  hipLaunchKernelGGL((KERN<MK, NW>), g, dim3(256), 0, stream, (const float*)x->data, (const float*)dz->data,            \
                     (const float*)(z ? z->data : nullptr), (float*)ws, a)
#define H3D_F32_BF_K(KERN)                                                                                              \
  do {                                                                                                                  \
    if (z && narrow) H3D_F32_BF(KERN, true, true);                                                                      \
    else if (z) H3D_F32_BF(KERN, true, false);                                                                          \
    else if (narrow) H3D_F32_BF(KERN, false, true);                                                                     \
    else H3D_F32_BF(KERN, false, false);                                                                                \
  } while (0)
  if (thin) H3D_F32_BF_K(bwd_filter_f32_thin_kernel);
  else H3D_F32_BF_K(bwd_filter_f32_mfma_kernel);
#undef H3D_F32_BF_K
#undef H3D_F32_BF
  const int64_t total = (int64_t)a.cout * a.cin * 28;
  hipLaunchKernelGGL(bwd_filter_f32_reduce_kernel, dim3((unsigned)cdiv(total, 16)), dim3(256), 0, stream, (const float*)ws, dw, db,
                     a.cin, a.cout, nchunks);
  note_kernel(handle, thin ? "bwd_filter_f32_mfma_kernel<thin>" : "bwd_filter_f32_mfma_kernel");
  return launch_status(handle, "conv3d_bwd_filter_f32_mfma");
}

}  // namespace h3d
