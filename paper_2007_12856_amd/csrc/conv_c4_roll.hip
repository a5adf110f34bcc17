// Row-streaming forward 3x3x3 convolution for the first layer (Cin <= 4, Cout <= 16, bf16), optionally fused with
// the 2x2x2 average pooling that follows it and with the sign mask of its activation (Sec. III-C "FP"; the layer is
// HBM-bound on paper, and the tile kernel in conv_small_cin.hip turned out to be bound by its LDS patch reads:
// 256 bytes of LDS per output voxel).
//
// Here the kh taps are folded into the accumulators and the two output planes of a wavefront share every MFMA:
//   * a wavefront owns TWO output planes x 64 columns and walks down the rows.  For an input row r and input plane
//     dz (four planes feed the two output planes), an A fragment (v_mfma_f32_32x32x16_bf16: 32 voxels x K = 16) holds,
//     per voxel, 4 column slots (kw = 0..2 and a zero-weight slot) x 4 channels: one 16-byte LDS read of two 8-byte
//     voxel units.  The 32 columns of the weight fragment are (output plane o, channel): plane o takes tap kd = dz - o
//     (zero where that is no tap), so one fragment read feeds both planes; it is multiplied by three weight
//     fragments, one per kh, into the accumulators of output rows r+1, r, r-1: 64 bytes of LDS per output voxel, and
//     no halo rows at all (every input row is staged once per workgroup);
//   * 4 planes x 3 kh = 12 MFMAs per 32 voxels and row for two output planes: 1.33 x the multiply count of the direct
//     form, on the tile shape that the matrix cores run at full rate (the 16x16x32 tile issues at 60 % of it);
//   * patches are the A operand, weights the B operand: an accumulator is four groups of four consecutive voxels of
//     one (plane, channel) per lane, so bias, activation and bf16 packing need no exchange; the 2x2x2 pooling adds
//     the two planes of a window, which sit in lanes l and l ^ 16: eight lane exchanges per 32 voxels and row pair,
//     after which each of the two lanes finishes half of the windows; rows that are stored (z, mask) go through a
//     per-wavefront LDS patch to leave as whole 16-byte pieces;
//   * the workgroup (4 wavefronts = 4 planes x 128 columns) keeps the six input planes of three consecutive rows in
//     an LDS ring: row t is multiplied while row t+2 is transposed in (channel-interleaved, 8 bytes per voxel) and
//     the loads of row t+3 are in flight; one LDS-only barrier per row.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
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
constexpr int CR_OTP = 64 + 8;                // output patch pitch (bf16 elements): 2 planes x 16 channels x 64 columns per wavefront
constexpr int CR_OOB = (int)0x80000000;
constexpr size_t CR_LDS_BYTES = (size_t)CR_RING * CR_SLOT * 8 + 4 * 32 * CR_OTP * 2;
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

// wp: [dz*3 + kh][lane][8] bf16 (B operand, 32x32x16): lane l = (column n = l % 32 = 16 o + co, k group kp = l / 32);
// input plane dz = 0..3 of the four that feed the output plane pair, tap kd = dz - o; element e: kw = 2 kp + e / 4,
// channel e % 4.  Zero for kd outside 0..2, kw > 2, channel >= Cin, co >= Cout.
__global__ void pack_w_c4_roll_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 12 * 512) return;
  const int e = i & 7, lane = (i >> 3) & 63, f = i >> 9;
  const int dz = f / 3, kh = f % 3;
  const int co = lane & 15, o = (lane >> 4) & 1, kp = lane >> 5;
  const int kd = dz - o, kw = 2 * kp + (e >> 2), ci = e & 3;
  bf16_t v = 0;
  if (kd >= 0 && kd < 3 && kw < 3 && ci < cin && co < cout) v = w[((int64_t)co * cin + ci) * 27 + kd * 9 + kh * 3 + kw];
  wp[i] = v;
}

__device__ __forceinline__ void cr_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// MAXF: 0 <= slope <= 1, so the activation is max(y, slope * y)
template <bool POOL, bool MAXF>
__global__ void __launch_bounds__(256, 2) conv3d_fwd_c4_roll_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                    const float* __restrict__ bias, bf16_t* __restrict__ out,
                                                                    C4RollArgs a) {
  extern __shared__ uint4 lds_raw[];
  uint2* ring = reinterpret_cast<uint2*>(lds_raw);                                             // [slot][plane][unit]
  bf16_t* ot_all = reinterpret_cast<bf16_t*>(ring + CR_RING * CR_SLOT);                        // [wave][16][CR_OTP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lj = lane & 15, lo = (lane >> 4) & 1, lh = lane >> 5;   // channel, plane of the pair, half of the k range / voxel sub-group
  const int W = a.in.w, H = a.in.h;
  int t0 = blockIdx.x;
  const int tw = t0 % a.tiles_w; t0 /= a.tiles_w;
  const int seg = t0 % a.segs; t0 /= a.segs;
  const int td = t0 % a.tiles_d;
  const int n = t0 / a.tiles_d;
  const int w0 = tw * CR_TW, ps0 = td * CR_TD;
  const int ha = seg * a.seg_rows, hb = min(H, ha + a.seg_rows);
  const int nsteps = hb - ha + 2;         // input rows ha-1 .. hb

  // ---- weights: twelve fragments (input plane dz, kh), registers for the whole kernel
  bf16x8 B[4][3];
#pragma unroll
  for (int dz = 0; dz < 4; ++dz)
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) B[dz][kh] = __builtin_bit_cast(bf16x8, wp[(dz * 3 + kh) * 64 + lane]);

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
  // A fragment (dz, vb): unit of staged plane 2 pp + dz, voxel w0 + 64 cp + 32 vb + lane % 32 + 2 lh - 1
  //                      = unit 64 cp + 32 vb + lane % 32 + 2 lh + 7
  int a_off[4];
#pragma unroll
  for (int dz = 0; dz < 4; ++dz) a_off[dz] = (2 * pp + dz) * CR_P + 64 * cp + (lane & 31) + 2 * lh + 7;
  const float bv = (bias && lj < a.cout) ? bias[lj] : 0.f;
  bf16_t* ot = ot_all + wave * 32 * CR_OTP;              // [plane of the pair][channel][column]
  const __amdgpu_buffer_rsrc_t rs_out = cr_rsrc(out ? out + n * a.out.nstride : in, out ? (uint32_t)a.out.nstride * 2 : 0u);
  // the sign mask alone (fused call that does not store z) comes straight from the registers: the two lanes that hold the
  // halves of every group of 8 voxels exchange one dword, and half of the lanes store 8 mask bytes (64 voxels of their
  // plane and channel) with one instruction; needs whole 8-byte pieces (W a multiple of 64, aligned mask)
  const bool mask_regs = a.mask && !out && (W % 64 == 0) && ((uintptr_t)a.mask % 8 == 0);
  const bool keep_row = out || (a.mask && !mask_regs);

  // accumulators [voxel block of 32][output row r+1, r, r-1]; register 4 j + i = voxel 32 vb + 8 j + 4 lh + i of
  // (plane lo, channel lj)
  f32x16 acc[2][3];
#pragma unroll
  for (int vb = 0; vb < 2; ++vb)
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[vb][k][r] = 0.f;
  float pa[2][4][2];         // POOL: pair sums (along W) of this lane's plane, first row of the window (plane 0: both rows
                             // once the second one is there), kept so that the window is added in the order of the separate
                             // pooling kernel: ((p0r0 + p0r1) + p1r0) + p1r1

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

  // One row step.  ROT = t % 3 is a compile-time constant (the loop below is unrolled three times), so the ring slots and
  // the three accumulator sets rotate by renaming: set (t - k) % 3 collects output row ha + t - k, nothing is moved.
  auto step = [&](auto rot_c, int t) {
    constexpr int ROT = decltype(rot_c)::value;
    constexpr int S0 = ROT, S1 = (ROT + 2) % 3, S2 = (ROT + 1) % 3;    // accumulator sets of kh = 0, 1, 2
    const uint2* rowp = ring + ROT * CR_SLOT;
    // ---- MFMAs of input row ha - 1 + t: contributions to output rows ha + t (kh = 0), ha + t - 1, ha + t - 2
#pragma unroll
    for (int vb = 0; vb < 2; ++vb) {
      bf16x8 A[4];
#pragma unroll
      for (int dz = 0; dz < 4; ++dz) {
        const uint2* p = rowp + a_off[dz] + 32 * vb;
        const uint2 u0 = p[0], u1 = p[1];
        const uint4 f = {u0.x, u0.y, u1.x, u1.y};
        A[dz] = __builtin_bit_cast(bf16x8, f);
      }
      // kh = 0 opens output row ha + t: its chain starts from zero (the set was read out two steps ago)
      {
        f32x16 zero;
#pragma unroll
        for (int r = 0; r < 16; ++r) zero[r] = 0.f;
        acc[vb][S0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[0], B[0][0], zero, 0, 0, 0);
      }
#pragma unroll
      for (int dz = 1; dz < 4; ++dz) acc[vb][S0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[dz], B[dz][0], acc[vb][S0], 0, 0, 0);
#pragma unroll
      for (int dz = 0; dz < 4; ++dz) {
        acc[vb][S1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[dz], B[dz][1], acc[vb][S1], 0, 0, 0);
        acc[vb][S2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[dz], B[dz][2], acc[vb][S2], 0, 0, 0);
      }
    }
    // ---- row t + 2 goes into the slot that row t - 1 has just left; then the loads of row t + 3
    if (t + 2 < nsteps) write(v, (ROT + 2) % 3);
    if (t + 3 < nsteps) issue(v, t + 3);

    // ---- output row ha + t - 2 is complete (accumulator [2]): bias, activation, store / mask / pooling
    if (t >= 2) {
      const int h = ha + t - 2;
      float cur[2][4][2];    // POOL: this row's pair sums
      uint32_t mbits = 0;    // mask_regs: nibble 4 vb + j = signs of this lane's four voxels of group (vb, j)
      asm volatile("" ::: "memory");
#pragma unroll
      for (int vb = 0; vb < 2; ++vb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float r[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            r[k] = acc[vb][S2][4 * j + k] + bv;
            if (MAXF) r[k] = fmaxf(r[k], r[k] * a.out_slope);
            else if (!(r[k] > 0.f)) r[k] *= a.out_slope;
          }
          const uint2 pk = {pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3])};
          if (keep_row) *reinterpret_cast<uint2*>(&ot[(16 * lo + lj) * CR_OTP + 32 * vb + 8 * j + 4 * lh]) = pk;
          if (mask_regs) {
            const uint32_t nib = ((int)(pk.x << 16) > 0 ? 1u : 0u) | ((int)(pk.x & 0xffff0000u) > 0 ? 2u : 0u) |
                                 ((int)(pk.y << 16) > 0 ? 4u : 0u) | ((int)(pk.y & 0xffff0000u) > 0 ? 8u : 0u);
            mbits |= nib << (4 * (4 * vb + j));
          }
          if (POOL) {
            // the pooling reads the values as they are stored (rounded to bf16), pairs along W first
            cur[vb][j][0] = __uint_as_float(pk.x << 16) + __uint_as_float(pk.x & 0xffff0000u);
            cur[vb][j][1] = __uint_as_float(pk.y << 16) + __uint_as_float(pk.y & 0xffff0000u);
          }
        }
      asm volatile("" ::: "memory");
      if (keep_row) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int u = lane + 64 * i;
          const int o = u >> 7, co = (u >> 3) & 15, wu = u & 7;
          const int ps = ps0 + 2 * pp + o;
          const int w = w0 + 64 * cp + 8 * wu;
          const uint4 q = *reinterpret_cast<const uint4*>(&ot[(16 * o + co) * CR_OTP + 8 * wu]);
          const bool ok = co < a.cout && w < W && ps < a.out.ds;
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
      if (mask_regs) {
        const uint32_t other = (uint32_t)__shfl_xor((int)mbits, 32, 64);
        const uint32_t lo_n = lh ? other : mbits, hi_n = lh ? mbits : other;     // low / high nibble of every byte
        auto spread = [](uint32_t x) {       // four nibbles -> the low nibbles of four bytes
          x &= 0xffffu;
          x = (x | (x << 8)) & 0x00ff00ffu;
          return (x | (x << 4)) & 0x0f0f0f0fu;
        };
        const uint2 mb = {spread(lo_n) | (spread(hi_n) << 4), spread(lo_n >> 16) | (spread(hi_n >> 16) << 4)};
        const int ps = ps0 + 2 * pp + lo;
        if (lh == 0 && lj < a.cout && ps < a.out.ds && w0 + 64 * cp < W)
          *reinterpret_cast<uint2*>(a.mask + ((((int64_t)n * a.cout + lj) * a.out.ds + ps) * H + h) * (W / 8) + ((w0 + 64 * cp) >> 3)) = mb;
      }
      if (POOL) {
        if (!(h & 1)) {
#pragma unroll
          for (int vb = 0; vb < 2; ++vb)
#pragma unroll
            for (int j = 0; j < 4; ++j) { pa[vb][j][0] = cur[vb][j][0]; pa[vb][j][1] = cur[vb][j][1]; }
        } else {
          // plane 0 lanes finish the windows of groups j = 0, 1, plane 1 lanes (l ^ 16) those of j = 2, 3
          const bool store_ok = ps0 + 2 * pp < a.out.ds && lj < a.cout;
          bf16_t* yo = a.ypool + n * a.yp.nstride + (int64_t)lj * a.yp.cstride + (int64_t)(((ps0 + 2 * pp) >> 1) + a.yp.hlo) * a.yp.plane +
                       (int64_t)(h >> 1) * (W >> 1) + ((w0 + 64 * cp) >> 1) + 2 * lh;
#pragma unroll
          for (int vb = 0; vb < 2; ++vb) {
            float x0[4][2];      // plane 0: p0r0 + p0r1
#pragma unroll
            for (int j = 0; j < 4; ++j) { x0[j][0] = pa[vb][j][0] + cur[vb][j][0]; x0[j][1] = pa[vb][j][1] + cur[vb][j][1]; }
            float res[2][2];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
              for (int s2 = 0; s2 < 2; ++s2) {
                // plane 0 lanes send their sum of group 2 + jj and receive plane 1's two rows of group jj; plane 1 lanes
                // send their two rows of group jj and receive plane 0's sum of group 2 + jj
                const float send_a = lo ? pa[vb][jj][s2] : x0[2 + jj][s2];
                const float send_b = lo ? cur[vb][jj][s2] : 0.f;
                const float got_a = __shfl_xor(send_a, 16, 64);
                const float got_b = __shfl_xor(send_b, 16, 64);
                res[jj][s2] = lo ? (got_a + pa[vb][2 + jj][s2]) + cur[vb][2 + jj][s2] : (x0[jj][s2] + got_a) + got_b;
              }
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
              const int j = 2 * lo + jj;
              if (store_ok && w0 + 64 * cp + 32 * vb + 8 * j + 4 * lh < W)
                *reinterpret_cast<uint32_t*>(yo + 16 * vb + 4 * j) = pack_bf16x2(res[jj][0] * 0.125f, res[jj][1] * 0.125f);
            }
          }
        }
      }
    }
    cr_barrier();
  };
  for (int t = 0; t < nsteps; t += 3) {
    step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < nsteps) step(std::integral_constant<int, 1>{}, t + 1);
    if (t + 2 < nsteps) step(std::integral_constant<int, 2>{}, t + 2);
  }
}

template <bool POOL, bool MAXF>
h3d_status launch_c4_roll(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, const h3d_tensor* y,
                          void* mask, float out_slope, void* ws, hipStream_t stream) {
  C4RollArgs a;
  a.in = make_geo(in); a.out = make_geo(z);
  a.yp = y ? make_geo(y) : a.out;
  a.cin = in->c; a.cout = z->c; a.out_slope = out_slope;
  a.ypool = y ? (bf16_t*)y->data : nullptr;
  a.mask = (uint8_t*)mask;
  auto kern = conv3d_fwd_c4_roll_kernel<POOL, MAXF>;
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
  hipLaunchKernelGGL(pack_w_c4_roll_kernel, dim3(24), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, a.cin, a.cout);
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

size_t c4_roll_ws_bytes() { return 12 * 512 * sizeof(bf16_t); }

h3d_status conv3d_fwd_c4_roll(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, const h3d_tensor* y,
                              void* mask, float out_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (!ws || ws_bytes < c4_roll_ws_bytes()) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace must be 16-byte aligned");
  if ((int64_t)z->n * z->d * z->h * z->w == 0) return H3D_OK;
  const bool maxf = out_slope >= 0.f && out_slope <= 1.f;
  if (y) return maxf ? launch_c4_roll<true, true>(handle, in, w, bias, z, y, mask, out_slope, ws, stream)
                     : launch_c4_roll<true, false>(handle, in, w, bias, z, y, mask, out_slope, ws, stream);
  return maxf ? launch_c4_roll<false, true>(handle, in, w, bias, z, nullptr, mask, out_slope, ws, stream)
              : launch_c4_roll<false, false>(handle, in, w, bias, z, nullptr, mask, out_slope, ws, stream);
}

}  // namespace h3d
