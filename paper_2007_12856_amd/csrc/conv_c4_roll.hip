// Row-streaming forward 3x3x3 convolution for the first layer (Cin <= 4, Cout <= 16, bf16), optionally fused with
// the 2x2x2 average pooling that follows it and with the sign mask of its activation (Sec. III-C "FP"; the layer is
// HBM-bound on paper, and the tile kernel in conv_small_cin.hip turned out to be bound by its LDS patch reads:
// 256 bytes of LDS per output voxel).
//
// Here the kh taps are folded into the accumulators and the kd taps are paired in the contraction:
//   * a wavefront owns TWO output planes x 64 columns and walks down the rows.  For an input row r, an A fragment
//     (v_mfma_f32_16x16x32_bf16: 16 voxels x K = 32) holds, per voxel, 2 input planes x 4 column slots (kw = 0..2 and
//     a zero-weight slot) x 4 channels: two 16-byte LDS reads of 8-byte voxel units.  The same fragment is multiplied
//     by three weight fragments, one per kh, into the accumulators of output rows r+1, r, r-1: 128 bytes of LDS per
//     output voxel, and no halo rows at all (every input row is staged once per workgroup);
//   * output plane o of the pair uses input planes o, o+1 (kd = 0, 1) in one fragment and o+2 (kd = 2, other half
//     zero) in a second: 2 x 3 MFMAs per 16 voxels, row and plane: 1.5 x the MFMA count of the direct form;
//   * patches are the A operand, weights the B operand: an accumulator is four consecutive voxels of one channel per
//     lane, so bias, activation, bf16 packing and the 2x2x2 pooling sums (both planes and both rows of a window
//     pass through the same lane) need no exchange; rows that are stored (z, mask) go through a per-wavefront LDS
//     patch to leave as whole 16-byte pieces;
//   * the workgroup (4 wavefronts = 4 planes x 128 columns) keeps the six input planes of three consecutive rows in
//     an LDS ring: row t is multiplied while row t+2 is transposed in (channel-interleaved, 8 bytes per voxel) and
//     the loads of row t+3 are in flight; one LDS-only barrier per row.
#include <algorithm>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int CR_TD = 4, CR_TW = 128;
constexpr int CR_NPL = CR_TD + 2;
constexpr int CR_XW = CR_TW + 16;             // staged row: columns w0-8 .. w0+TW+7, one 8-byte unit (4 channels) per voxel
constexpr int CR_P = CR_XW + 2;               // plane pitch inside a ring slot (units)
constexpr int CR_SLOT = CR_NPL * CR_P;        // units per ring slot
constexpr int CR_RING = 3;
constexpr int CR_NG = CR_XW / 8;              // column groups of 8 per row
constexpr int CR_ITEMS = CR_NPL * CR_NG;      // staging items of a row: (plane, group of 8 columns)
constexpr int CR_OTP = 64 + 8;                // output patch pitch (bf16 elements): 16 channels x 64 columns per wavefront
constexpr int CR_OOB = (int)0x80000000;
constexpr size_t CR_LDS_BYTES = (size_t)CR_RING * CR_SLOT * 8 + 4 * 16 * CR_OTP * 2;
static_assert(CR_ITEMS <= 256, "one staging item per lane");

struct C4RollArgs {
  Geo in, out, yp;
  int cin, cout;
  int tiles_w, tiles_d, segs, seg_rows;
  float out_slope;
  bf16_t* ypool;       // pooled output (POOL)
  uint8_t* mask;       // sign mask or NULL: bit k of byte j of a row = stored value of voxel 8 j + k is > 0
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t cr_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                           (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

// wp: [t*3 + kh][lane][8] bf16 (B operand, 16x16x32): lane l = (co = l % 16, k group g = l / 16); g = 2 ph + kp:
// plane half ph (kd = 2 t + ph), column pair kp; element e: kw = 2 kp + e / 4, channel e % 4.  Zero for kd > 2,
// kw > 2, channel >= Cin, co >= Cout.
__global__ void pack_w_c4_roll_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 6 * 512) return;
  const int e = i & 7, lane = (i >> 3) & 63, f = i >> 9;
  const int t = f / 3, kh = f % 3;
  const int co = lane & 15, g = lane >> 4, ph = g >> 1, kp = g & 1;
  const int kd = 2 * t + ph, kw = 2 * kp + (e >> 2), ci = e & 3;
  bf16_t v = 0;
  if (kd < 3 && kw < 3 && ci < cin && co < cout) v = w[((int64_t)co * cin + ci) * 27 + kd * 9 + kh * 3 + kw];
  wp[i] = v;
}

__device__ __forceinline__ void cr_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <bool POOL>
__global__ void __launch_bounds__(256, 2) conv3d_fwd_c4_roll_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                    const float* __restrict__ bias, bf16_t* __restrict__ out,
                                                                    C4RollArgs a) {
  extern __shared__ uint4 lds_raw[];
  uint2* ring = reinterpret_cast<uint2*>(lds_raw);                                             // [slot][plane][unit]
  bf16_t* ot_all = reinterpret_cast<bf16_t*>(ring + CR_RING * CR_SLOT);                        // [wave][16][CR_OTP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lj = lane & 15;
  const int W = a.in.w, H = a.in.h;
  int t0 = blockIdx.x;
  const int tw = t0 % a.tiles_w; t0 /= a.tiles_w;
  const int seg = t0 % a.segs; t0 /= a.segs;
  const int td = t0 % a.tiles_d;
  const int n = t0 / a.tiles_d;
  const int w0 = tw * CR_TW, ps0 = td * CR_TD;
  const int ha = seg * a.seg_rows, hb = min(H, ha + a.seg_rows);
  const int nsteps = hb - ha + 2;         // input rows ha-1 .. hb

  // ---- weights: six fragments (kd pair t, kh), registers for the whole kernel
  bf16x8 B[2][3];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) B[t][kh] = __builtin_bit_cast(bf16x8, wp[(t * 3 + kh) * 64 + lane]);

  // ---- staging role: item = (input plane, group of 8 columns): 4 loads of 16 bytes (one per channel), 16 byte-permutes,
  //      four 16-byte LDS stores (8 voxel units of 8 bytes)
  const int item = tid;
  const int sgrp = item % CR_NG, sdz = item / CR_NG;
  const __amdgpu_buffer_rsrc_t rs_in = cr_rsrc(in + n * a.in.nstride, (uint32_t)a.in.nstride * 2);
  bool st_ok;
  int st_base;
  {
    const int p_in = ps0 - a.out.hlo + sdz - 1;       // local interior index of the input plane
    const int64_t gq = a.in.doff + p_in;
    const int sp = p_in + a.in.hlo;
    const int wc = w0 - 8 + 8 * sgrp;
    st_ok = item < CR_ITEMS && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && wc >= 0 && wc + 8 <= W;
    st_base = 2 * (sp * (int)a.in.plane + wc);
  }
  const int st_dst = sdz * CR_P + 8 * sgrp;            // first of the item's 8 units inside a ring slot
  auto issue = [&](u32x4 (&v)[4], int t) {             // global loads of input row ha - 1 + t
    const int h = ha - 1 + t;
    const int vo = (st_ok && h >= 0 && h < H && t < nsteps) ? st_base + 2 * h * W : CR_OOB;
#pragma unroll
    for (int ci = 0; ci < 4; ++ci)
      v[ci] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, ci < a.cin ? vo : CR_OOB, __builtin_amdgcn_readfirstlane(2 * ci * (int)a.in.cstride), 0);
  };
  auto write = [&](const u32x4 (&v)[4], int slot) {    // channel-interleave 8 voxels into the ring
    if (item >= CR_ITEMS) return;
    uint4* dst = reinterpret_cast<uint4*>(ring + slot * CR_SLOT + st_dst);
#pragma unroll
    for (int k = 0; k < 4; ++k) {                      // voxels 2k and 2k+1 of the group
      uint4 u;
      u.x = __builtin_amdgcn_perm(v[1][k], v[0][k], 0x05040100);
      u.y = __builtin_amdgcn_perm(v[3][k], v[2][k], 0x05040100);
      u.z = __builtin_amdgcn_perm(v[1][k], v[0][k], 0x07060302);
      u.w = __builtin_amdgcn_perm(v[3][k], v[2][k], 0x07060302);
      dst[k] = u;
    }
  };

  // ---- compute role: output planes ps0 + 2 pp + {0, 1}, columns w0 + 64 cp .. + 63
  const int pp = wave >> 1, cp = wave & 1;
  const int ph = lg >> 1, kp = lg & 1;
  // A fragment (o, t): unit of input plane dz = 2 pp + o + 2 t + ph (the zero-weight half of t = 1 reads plane dz - 1
  // again: any staged plane will do), voxel w0 + 64 cp + 16 vb + lj + 2 kp - 1 = unit 64 cp + 16 vb + lj + 2 kp + 7
  int a_off[2][2];
#pragma unroll
  for (int o = 0; o < 2; ++o)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      int dz = 2 * pp + o + 2 * t + ph;
      if (t == 1 && ph == 1) dz -= 1;
      a_off[o][t] = dz * CR_P + 64 * cp + lj + 2 * kp + 7;
    }
  const float bv = (bias && lj < a.cout) ? bias[lj] : 0.f;
  bf16_t* ot = ot_all + wave * 16 * CR_OTP;
  const __amdgpu_buffer_rsrc_t rs_out = cr_rsrc(out ? out + n * a.out.nstride : in, out ? (uint32_t)a.out.nstride * 2 : 0u);
  const bool keep_row = out || a.mask;

  f32x4 acc[2][4][3];        // [plane of the pair][voxel block][output row r+1, r, r-1]
#pragma unroll
  for (int o = 0; o < 2; ++o)
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
      for (int k = 0; k < 3; ++k) acc[o][vb][k] = f32x4{0.f, 0.f, 0.f, 0.f};
  float pa[2][4][2];         // POOL: pair sums of the window's first row, per plane (kept so that the window is added in
                             // the order of the separate pooling kernel)

  // ---- prologue: rows 0 and 1 into the ring, row 2 in flight
  u32x4 v[4];
  {
    u32x4 v1[4];
    issue(v, 0);
    issue(v1, 1);
    write(v, 0);
    write(v1, 1);
  }
  issue(v, 2);
  cr_barrier();

  int slot = 0;
  for (int t = 0; t < nsteps; ++t) {
    const uint2* rowp = ring + slot * CR_SLOT;
    // ---- MFMAs of input row ha - 1 + t: contributions to output rows ha + t (kh = 0), ha + t - 1, ha + t - 2
#pragma unroll
    for (int vb = 0; vb < 4; ++vb) {
      bf16x8 A[2][2];
#pragma unroll
      for (int o = 0; o < 2; ++o)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const uint2* p = rowp + a_off[o][tt] + 16 * vb;
          const uint2 lo = p[0], hi = p[1];
          const uint4 f = {lo.x, lo.y, hi.x, hi.y};
          A[o][tt] = __builtin_bit_cast(bf16x8, f);
        }
#pragma unroll
      for (int o = 0; o < 2; ++o)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
          acc[o][vb][kh] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[o][0], B[0][kh], acc[o][vb][kh], 0, 0, 0);
          acc[o][vb][kh] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[o][1], B[1][kh], acc[o][vb][kh], 0, 0, 0);
        }
    }
    // ---- row t + 2 goes into the slot that row t - 1 has just left; then the loads of row t + 3
    if (t + 2 < nsteps) write(v, slot == 0 ? 2 : slot - 1);
    if (t + 3 < nsteps) issue(v, t + 3);

    // ---- output row ha + t - 2 is complete (accumulator [2]): bias, activation, store / mask / pooling
    if (t >= 2) {
      const int h = ha + t - 2;
#pragma unroll
      for (int o = 0; o < 2; ++o) {
        const int ps = ps0 + 2 * pp + o;
        const bool plane_ok = ps < a.out.ds;
        asm volatile("" ::: "memory");
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
          float r[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            r[k] = acc[o][vb][2][k] + bv;
            if (!(r[k] > 0.f)) r[k] *= a.out_slope;
          }
          const uint2 pk = {pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3])};
          if (keep_row) *reinterpret_cast<uint2*>(&ot[lj * CR_OTP + vb * 16 + 4 * lg]) = pk;
          if (POOL) {
            // the pooling reads the values as they are stored (rounded to bf16), pairs along W first
            const float s0 = __uint_as_float(pk.x << 16) + __uint_as_float(pk.x & 0xffff0000u);
            const float s1 = __uint_as_float(pk.y << 16) + __uint_as_float(pk.y & 0xffff0000u);
            if (!(h & 1)) {
              pa[o][vb][0] = s0; pa[o][vb][1] = s1;
            } else if (o == 0) {
              pa[0][vb][0] += s0; pa[0][vb][1] += s1;                 // plane 0: row 0 + row 1
            } else {
              // window order of the separate kernel: ((p0r0 + p0r1) + p1r0) + p1r1
              pa[0][vb][0] = (pa[0][vb][0] + pa[1][vb][0]) + s0;
              pa[0][vb][1] = (pa[0][vb][1] + pa[1][vb][1]) + s1;
            }
          }
        }
        asm volatile("" ::: "memory");
        if (keep_row && plane_ok) {
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int u = lane + 64 * i;
            const int co = u >> 3, wu = u & 7;
            const int w = w0 + 64 * cp + 8 * wu;
            const uint4 q = *reinterpret_cast<const uint4*>(&ot[co * CR_OTP + 8 * wu]);
            const bool ok = co < a.cout && w < W;
            if (out) {
              const int vo = ok ? 2 * (co * (int)a.out.cstride + ps * (int)a.out.plane + h * W + w) : CR_OOB;
              __builtin_amdgcn_raw_buffer_store_b128(u32x4{q.x, q.y, q.z, q.w}, rs_out, vo, 0, 0);
            }
            if (a.mask && ok) {
              const uint32_t e[4] = {q.x, q.y, q.z, q.w};
              uint32_t bits = 0;
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                bits |= ((int)(e[k] << 16) > 0 ? 1u : 0u) << (2 * k);
                bits |= ((int)(e[k] & 0xffff0000u) > 0 ? 1u : 0u) << (2 * k + 1);
              }
              a.mask[((((int64_t)n * a.cout + co) * a.out.ds + ps) * H + h) * (W / 8) + (w >> 3)] = (uint8_t)bits;
            }
          }
        }
      }
      if (POOL && (h & 1) && ps0 + 2 * pp < a.out.ds && lj < a.cout) {
        // the window is complete: scale, round, 4-byte stores of two pooled voxels
        bf16_t* yo = a.ypool + n * a.yp.nstride + (int64_t)lj * a.yp.cstride + (int64_t)(((ps0 + 2 * pp) >> 1) + a.yp.hlo) * a.yp.plane +
                     (int64_t)(h >> 1) * (W >> 1) + ((w0 + 64 * cp) >> 1) + 2 * lg;
#pragma unroll
        for (int vb = 0; vb < 4; ++vb)
          if (w0 + 64 * cp + 16 * vb + 4 * lg < W)
            *reinterpret_cast<uint32_t*>(yo + 8 * vb) = pack_bf16x2(pa[0][vb][0] * 0.125f, pa[0][vb][1] * 0.125f);
      }
    }
    // ---- slide: what was accumulated for output row r+1 now waits as row r, row r as row r-1
#pragma unroll
    for (int o = 0; o < 2; ++o)
#pragma unroll
      for (int vb = 0; vb < 4; ++vb) {
        acc[o][vb][2] = acc[o][vb][1];
        acc[o][vb][1] = acc[o][vb][0];
        acc[o][vb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    cr_barrier();
    slot = slot == CR_RING - 1 ? 0 : slot + 1;
  }
}

template <bool POOL>
h3d_status launch_c4_roll(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, const h3d_tensor* y,
                          void* mask, float out_slope, void* ws, hipStream_t stream) {
  C4RollArgs a;
  a.in = make_geo(in); a.out = make_geo(z);
  a.yp = y ? make_geo(y) : a.out;
  a.cin = in->c; a.cout = z->c; a.out_slope = out_slope;
  a.ypool = y ? (bf16_t*)y->data : nullptr;
  a.mask = (uint8_t*)mask;
  auto kern = conv3d_fwd_c4_roll_kernel<POOL>;
  static int wgs_per_cu = 0;
  if (wgs_per_cu == 0) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)CR_LDS_BYTES) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d_fwd: cannot set the dynamic LDS size to %zu bytes", CR_LDS_BYTES);
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 256, CR_LDS_BYTES) != hipSuccess || nb < 1) nb = 1;
    wgs_per_cu = nb;
  }
  a.tiles_w = (int)cdiv(z->w, CR_TW);
  a.tiles_d = (int)cdiv(a.out.ds, CR_TD);
  // row segments (an even number of rows each): enough of them to fill the resident workgroup slots in the fewest rounds
  const int64_t base = (int64_t)z->n * a.tiles_d * a.tiles_w;
  const int64_t slots = (int64_t)wgs_per_cu * static_cast<Handle*>(handle)->num_cu;
  int best = 1;
  int64_t best_cost = -1;
  for (int s = 1; s <= std::max(1, z->h / 8); ++s) {
    const int64_t rows = 2 * cdiv(cdiv(z->h, s), 2);
    const int64_t cost = cdiv(base * cdiv(z->h, rows), slots) * (rows + 5);
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = s; }
  }
  a.seg_rows = (int)(2 * cdiv(cdiv(z->h, best), 2));
  a.segs = (int)cdiv(z->h, a.seg_rows);
  const int64_t nwg = base * a.segs;
  if (nwg == 0) return H3D_OK;
  if (nwg >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_fwd: too many workgroups");
  hipLaunchKernelGGL(pack_w_c4_roll_kernel, dim3(12), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, a.cin, a.cout);
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(256), CR_LDS_BYTES, stream, (const bf16_t*)in->data, (const uint4*)ws, bias,
                     (bf16_t*)z->data, a);
  return launch_status(handle, "conv3d_fwd_c4_roll");
}

}  // namespace

// bf16, Cin <= 4, Cout <= 16, output without halos, W a multiple of 8, at least 8 rows, 16-byte-aligned tensors,
// 31-bit byte offsets inside a sample
bool c4_roll_supported(const h3d_tensor* in, const h3d_tensor* z) {
  if (in->dtype != H3D_BF16 || in->c < 1 || in->c > 4 || z->c < 1 || z->c > 16) return false;
  if (z->halo_lo || z->halo_hi || z->w % 8 || z->h < 8) return false;      // (plane-run views are fine: the kernel uses the strides)
  if ((uintptr_t)in->data % 16 || (z->data && (uintptr_t)z->data % 16)) return false;
  return sample_span(in) < ((int64_t)1 << 30) && (int64_t)z->c * z->d * z->h * z->w < ((int64_t)1 << 30);
}

size_t c4_roll_ws_bytes() { return 6 * 512 * sizeof(bf16_t); }

h3d_status conv3d_fwd_c4_roll(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, const h3d_tensor* y,
                              void* mask, float out_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (!ws || ws_bytes < c4_roll_ws_bytes()) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace must be 16-byte aligned");
  if ((int64_t)z->n * z->d * z->h * z->w == 0) return H3D_OK;
  return y ? launch_c4_roll<true>(handle, in, w, bias, z, y, mask, out_slope, ws, stream)
           : launch_c4_roll<false>(handle, in, w, bias, z, nullptr, mask, out_slope, ws, stream);
}

}  // namespace h3d
