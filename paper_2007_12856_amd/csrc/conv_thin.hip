// 3x3x3 convolution with very few OUTPUT channels (at most 8) and at most 16 input channels, bf16 on the
// matrix cores: the backward-data pass of a network's first layer (Sec. III-C "BD": dx of a 4-channel
// input from a 16-channel g), or a forward pass onto a handful of channels.
//
// With so few output channels the 32 rows of v_mfma_f32_32x32x16_bf16 would be almost empty, so the kh
// taps are folded into them: row 8 kh + m of the A operand holds the weights of output channel m under
// tap row kh.  One MFMA per (kd, kw) on an INPUT row then yields that row's contribution to three output
// rows at once; the accumulator slides down one tap row per input row (kh = 0 -> 1 -> 2) and the kh = 2
// quarter leaves as a finished output row.  9 MFMAs per input row instead of 27 per output row, and the
// nine weight fragments stay in registers for the whole workgroup.
//   * accumulator layout: lanes 0..31 hold rows 0-3, 8-11, 16-19 (kh = 0,1,2 of channels 0..3), lanes 32..63
//     rows 4-7, 12-15, 20-23 (channels 4..7): the slide is a register move, no cross-lane traffic;
//   * the input tile is transposed into LDS as 16-byte units of 8 channels, [ci-group][plane][row][w], as
//     in the general kernel, so the B operand of tap (kd, kw) is one ds_read_b128 per lane;
//   * a workgroup = 4 wavefronts = 4 output planes x 4 rows x 64 columns (two MFMA column blocks per
//     wavefront: two independent accumulator chains).
#include <algorithm>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int T_TD = 4, T_TH = 4, T_TW = 64;
constexpr int T_NU = 68;                                  // units of a row: unit u holds column w0 - 2 + u; 1..66 are used
// A row is stored as 8 interleaved sub-rows: unit u sits at t_pos(u + 1) = ((u + 1) % 8) * 9 + (u + 1) / 8.  The
// staging threads, which own whole groups of 8 columns, then write consecutive positions (no bank conflicts:
// lanes run over the column groups of a row, then over planes, whose pitch 6 * 71 = 10 (mod 16) continues the
// sequence), and the 16 lanes of a ds_read_b128 pass, which want consecutive units starting at u + 1 = 2..4
// (mod 8), still hit 16 distinct bank groups.  71 positions per row: two workgroups fill the CU's 160 KB exactly.
constexpr int T_P = 71;
__host__ __device__ constexpr int t_pos(int v) { return (v & 7) * 9 + (v >> 3); }
constexpr int T_PAIRS = T_NU / 2;
constexpr int T_CIG_UNITS = (T_TD + 2) * (T_TH + 2) * T_P;
constexpr int T_ITEMS = 2 * (T_TD + 2) * (T_TH + 2) * T_PAIRS;
constexpr int T_THREADS = 256;
constexpr int T_ROUNDS = (T_ITEMS + T_THREADS - 1) / T_THREADS;
constexpr int T_OOB = (int)0x80000000;

struct ThinArgs {
  Geo in, out;
  int cin_k, cout_k;
  int tiles_w, tiles_h, tiles_d;
  float out_slope;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t thin_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                           (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

// wp: [step = kd*3+kw][lane][8] bf16; lane l, element e: row 8 kh + m = l % 32 (kh < 3), input channel 8 (l/32) + e
__global__ void pack_w_thin_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout, int transpose) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 9 * 512) return;
  const int e = i & 7, lane = (i >> 3) & 63, step = i >> 9;
  const int kd = step / 3, kw = step % 3;
  const int row = lane & 31, kh = row >> 3, m = row & 7, c = (lane >> 5) * 8 + e;
  const int cin_k = transpose ? cout : cin, cout_k = transpose ? cin : cout;
  bf16_t v = 0;
  if (kh < 3 && m < cout_k && c < cin_k) {
    const int tap = kd * 9 + kh * 3 + kw;
    v = transpose ? w[((int64_t)c * cin + m) * 27 + (26 - tap)] : w[((int64_t)m * cin + c) * 27 + tap];
  }
  wp[i] = v;
}

template <bool VEC8>
__global__ void __launch_bounds__(T_THREADS, 2) conv3d_thin_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                   const float* __restrict__ bias, bf16_t* __restrict__ out,
                                                                   ThinArgs a) {
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63, wd = tid >> 6;
  const int W = a.in.w, H = a.in.h;
  // consecutive workgroup ids go to different XCDs (each with its own L2): hand every XCD a contiguous run
  // of tiles, so that tiles sharing halo rows and planes meet in one L2
  const int G = gridDim.x;
  int t = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  const int tw = t % a.tiles_w; t /= a.tiles_w;
  const int th = t % a.tiles_h; t /= a.tiles_h;
  const int td = t % a.tiles_d;
  const int n = t / a.tiles_d;
  const int w0 = tw * T_TW, h0 = th * T_TH, ps0 = td * T_TD;

  // ---- weights: nine fragments, resident in registers
  bf16x8 A[9];
#pragma unroll
  for (int s = 0; s < 9; ++s) A[s] = __builtin_bit_cast(bf16x8, wp[s * 64 + lane]);

  // ---- input tile -> LDS, transposed to units of 8 channels.
  if (VEC8) {
    // An item = (ci-group, plane, row, group of 8 columns): 8 loads of 16 bytes (one per channel), an 8 x 8
    // transpose by byte-permutes, up to eight 16-byte LDS stores.  Groups 0 and 9 only contribute the two
    // columns next to the tile (w0-2, w0-1 and w0+64, w0+65).
    const __amdgpu_buffer_rsrc_t rs_in = thin_rsrc(in + n * a.in.nstride, (uint32_t)a.in.nstride * 2);
    constexpr int NG = T_TW / 8 + 2;
    constexpr int ITEMS8 = 2 * (T_TD + 2) * (T_TH + 2) * NG;
    constexpr int ROUNDS8 = (ITEMS8 + T_THREADS - 1) / T_THREADS;
    // every load of the tile is issued before the first transpose, so one memory latency covers them all
    u32x4 v[ROUNDS8][8];
#pragma unroll
    for (int r = 0; r < ROUNDS8; ++r) {
      const int item = tid + r * T_THREADS;
      const int grp = item % NG;
      int q = item / NG;
      const int dz = q % (T_TD + 2); q /= (T_TD + 2);
      const int hy = q % (T_TH + 2);
      const int cig = q / (T_TH + 2);
      const int p_in = ps0 - a.out.hlo + dz - 1;
      const int64_t gq = a.in.doff + p_in;
      const int sp = p_in + a.in.hlo;
      const int h = h0 + hy - 1, w = w0 - 8 + 8 * grp;
      const bool ok = item < ITEMS8 && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H && w >= 0 && w + 8 <= W;
      const int base = 2 * (cig * 8 * (int)a.in.cstride + sp * (int)a.in.plane + h * W + w);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const bool chan_ok = cig * 8 + e < a.cin_k;
        v[r][e] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, (ok && chan_ok) ? base : T_OOB,
                                                        __builtin_amdgcn_readfirstlane(2 * e * (int)a.in.cstride), 0);
      }
    }
#pragma unroll
    for (int r = 0; r < ROUNDS8; ++r) {
      const int item = tid + r * T_THREADS;
      if (item >= ITEMS8) continue;
      const int grp = item % NG;
      int q = item / NG;
      const int dz = q % (T_TD + 2); q /= (T_TD + 2);
      const int hy = q % (T_TH + 2);
      const int cig = q / (T_TH + 2);
      // this group's column c is unit u = 8 grp - 6 + c, and u + 1 = 8 (grp - 1) + (c + 3)
      uint4* dst = lds + (cig * (T_TD + 2) + dz) * ((T_TH + 2) * T_P) + hy * T_P + grp - 1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {       // dword j of each channel = columns 2j, 2j+1 of the group
        uint4 u0, u1;
        u0.x = __builtin_amdgcn_perm(v[r][1][j], v[r][0][j], 0x05040100); u1.x = __builtin_amdgcn_perm(v[r][1][j], v[r][0][j], 0x07060302);
        u0.y = __builtin_amdgcn_perm(v[r][3][j], v[r][2][j], 0x05040100); u1.y = __builtin_amdgcn_perm(v[r][3][j], v[r][2][j], 0x07060302);
        u0.z = __builtin_amdgcn_perm(v[r][5][j], v[r][4][j], 0x05040100); u1.z = __builtin_amdgcn_perm(v[r][5][j], v[r][4][j], 0x07060302);
        u0.w = __builtin_amdgcn_perm(v[r][7][j], v[r][6][j], 0x05040100); u1.w = __builtin_amdgcn_perm(v[r][7][j], v[r][6][j], 0x07060302);
        const int u = 8 * grp - 6 + 2 * j;
        if (u >= 1 && u <= T_NU - 2) dst[t_pos(2 * j + 3)] = u0;
        if (u + 1 >= 1 && u + 1 <= T_NU - 2) dst[t_pos(2 * j + 4)] = u1;
      }
    }
  } else {
    // An item = (ci-group, plane, row, pair of columns): 8 dword loads (one per channel, two voxels each),
    // 8 byte-permutes, two 16-byte LDS stores.
    const __amdgpu_buffer_rsrc_t rs_in = thin_rsrc(in + n * a.in.nstride, (uint32_t)a.in.nstride * 2);
    constexpr int HALF = (T_ROUNDS + 1) / 2;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      uint32_t v[HALF][8];
      int unit[HALF], upair[HALF];   // LDS row base and first unit of the pair
#pragma unroll
      for (int rr = 0; rr < HALF; ++rr) {
        const int r = half * HALF + rr;
        const int item = tid + r * T_THREADS;
        const int pair = item % T_PAIRS;
        int q = item / T_PAIRS;
        const int hy = q % (T_TH + 2); q /= (T_TH + 2);
        const int dz = q % (T_TD + 2);
        const int cig = q / (T_TD + 2);
        const bool item_ok = r < T_ROUNDS && item < T_ITEMS;
        unit[rr] = item_ok ? (cig * (T_TD + 2) + dz) * ((T_TH + 2) * T_P) + hy * T_P : -1;
        upair[rr] = 2 * pair;
        const int p_in = ps0 - a.out.hlo + dz - 1;        // local interior index of the input plane
        const int64_t gq = a.in.doff + p_in;
        const int sp = p_in + a.in.hlo;
        const int h = h0 + hy - 1, w = w0 - 2 + 2 * pair;
        const bool ok = item_ok && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H && w >= 0 && w + 1 < W;
        const int base = 2 * (cig * 8 * (int)a.in.cstride + sp * (int)a.in.plane + h * W + w);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool chan_ok = cig * 8 + e < a.cin_k;
          v[rr][e] = __builtin_amdgcn_raw_buffer_load_b32(rs_in, (ok && chan_ok) ? base : T_OOB,
                                                         __builtin_amdgcn_readfirstlane(2 * e * (int)a.in.cstride), 0);
        }
      }
#pragma unroll
      for (int rr = 0; rr < HALF; ++rr) {
        if (unit[rr] < 0) continue;
        const uint32_t* g = v[rr];
        uint4 u0, u1;   // unit of w (low halves) and of w+1 (high halves): 8 channels each
        u0.x = __builtin_amdgcn_perm(g[1], g[0], 0x05040100); u1.x = __builtin_amdgcn_perm(g[1], g[0], 0x07060302);
        u0.y = __builtin_amdgcn_perm(g[3], g[2], 0x05040100); u1.y = __builtin_amdgcn_perm(g[3], g[2], 0x07060302);
        u0.z = __builtin_amdgcn_perm(g[5], g[4], 0x05040100); u1.z = __builtin_amdgcn_perm(g[5], g[4], 0x07060302);
        u0.w = __builtin_amdgcn_perm(g[7], g[6], 0x05040100); u1.w = __builtin_amdgcn_perm(g[7], g[6], 0x07060302);
        if (upair[rr] >= 1) lds[unit[rr] + t_pos(upair[rr] + 1)] = u0;
        if (upair[rr] + 1 <= T_NU - 2) lds[unit[rr] + t_pos(upair[rr] + 2)] = u1;
      }
    }
  }
  __syncthreads();

  // ---- this wavefront: output plane ps0 + wd, rows h0 .. h0+3, columns w0 .. w0+63
  const int ps = ps0 + wd;
  const int half = lane >> 5, col = lane & 31;
  const bool plane_stored = ps < a.out.ds;
  const int64_t gp = a.out.doff + ps - a.out.hlo;
  const bool inside = gp >= 0 && gp < a.out.dglob;          // planes outside the global volume are written as zeros
  const __amdgpu_buffer_rsrc_t rs_out = thin_rsrc(out + n * a.out.nstride, (uint32_t)a.out.nstride * 2);
  float bv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bv[i] = (bias && 4 * half + i < a.cout_k) ? bias[4 * half + i] : 0.f;

  const uint4* base = lds + half * T_CIG_UNITS + wd * ((T_TH + 2) * T_P);
  int lane_pos[3];      // position of unit u = col + 1 + kw inside a row (column block 1 lies 4 positions on)
#pragma unroll
  for (int kw = 0; kw < 3; ++kw) lane_pos[kw] = t_pos(col + 2 + kw);
  f32x16 acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

  // B fragments are read two (kd, kw) steps ahead of the MFMAs that use them
  constexpr int NSTEP = (T_TH + 2) * 9;
  auto frag = [&](int step, int cb) {
    const int hi = step / 9, kd = (step % 9) / 3, kw = step % 3;
    return base[(kd * (T_TH + 2) + hi) * T_P + cb * 4 + lane_pos[kw]];
  };
  uint4 bq[3][2];
#pragma unroll
  for (int s0 = 0; s0 < 2; ++s0)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) bq[s0][cb] = frag(s0, cb);
#pragma unroll
  for (int hi = 0; hi < T_TH + 2; ++hi) {
    // slide: what was accumulated under tap row kh now waits for tap row kh + 1 of the next input row
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[cb][8 + i] = acc[cb][4 + i];
        acc[cb][4 + i] = acc[cb][i];
        acc[cb][i] = 0.f;
      }
#pragma unroll
    for (int k9 = 0; k9 < 9; ++k9) {
      const int step = hi * 9 + k9;
      if (step + 2 < NSTEP) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) bq[(step + 2) % 3][cb] = frag(step + 2, cb);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[k9], __builtin_bit_cast(bf16x8, bq[step % 3][cb]), acc[cb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (hi >= 2 && plane_stored) {
      const int h = h0 + hi - 2;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const int w = w0 + cb * 32 + col;
        const int vo = (h < H && w < W) ? 2 * (4 * half * (int)a.out.cstride + ps * (int)a.out.plane + h * W + w) : T_OOB;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float val = acc[cb][8 + i] + bv[i];
          if (!(val > 0.f)) val *= a.out_slope;
          const bool ch_ok = 4 * half + i < a.cout_k;
          __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16(inside ? val : 0.f), rs_out, ch_ok ? vo : T_OOB,
                                                __builtin_amdgcn_readfirstlane(2 * i * (int)a.out.cstride), 0);
        }
      }
    }
  }
}


// ---------------------------------------------------------------------------------------------------------
// Row-streaming variant for at most 4 output channels (the first layer's backward-data pass).
//
// The tap-row folding makes the accumulator walk down the rows by itself, so a workgroup does not need a
// tile of rows at all: it owns 4 output planes x 64 columns and streams along H.  Per input row it keeps the
// six planes of that row in an LDS ring of three rows (41 KB: three workgroups per CU), computes on row t
// while row t+2 is being transposed into the ring and the global loads of rows t+3, t+4 are in flight.
//   * no row halo: every input row is staged once per workgroup and its 9-tap MFMAs are issued once;
//   * with <= 4 output channels the 32 MFMA rows hold TWO output planes: row 8 kh + 4 o + m is channel m of
//     plane o under tap row kh, and the A fragment of input plane dz carries tap kd = dz - o in the rows of
//     plane o.  A wavefront = 2 planes x 32 columns, 12 MFMAs (4 input planes x 3 kw) per row, and the two
//     lane halves of the accumulator are the two planes, so every lane stores in the epilogue;
//   * wavefront pairs take turns staging: pair j owns the rows t = j (mod 2), one item (ci-group, plane,
//     group of 8 columns: 8 loads, 32 byte-permutes, 8 LDS stores) per lane.
constexpr int R_TD = 4;
constexpr int R_NPL = R_TD + 2;
constexpr int R_SLOT = 2 * R_NPL * T_P;        // 16-byte units of one ring slot: [ci-group][plane][position]
constexpr int R_RING = 3;
constexpr int R_NG = T_TW / 8 + 2;
constexpr int R_ITEMS = 2 * R_NPL * R_NG;      // staging items of a row
static_assert(R_ITEMS <= 128, "one item per lane of a wavefront pair");

struct ThinRollArgs {
  Geo in, out;
  int cin_k, cout_k;
  int tiles_w, tiles_d, segs, seg_rows;
  float out_slope;
};

// wp: [dz*3 + kw][lane][8] bf16; lane l, element e: row l % 32 = 8 kh + 4 o + m, input channel 8 (l/32) + e,
// depth tap kd = dz - o
__global__ void pack_w_thin_roll_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout, int transpose) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 12 * 512) return;
  const int e = i & 7, lane = (i >> 3) & 63, step = i >> 9;
  const int dz = step / 3, kw = step % 3;
  const int row = lane & 31, kh = row >> 3, o = (row >> 2) & 1, m = row & 3, c = (lane >> 5) * 8 + e;
  const int kd = dz - o;
  const int cin_k = transpose ? cout : cin, cout_k = transpose ? cin : cout;
  bf16_t v = 0;
  if (kh < 3 && kd >= 0 && kd < 3 && m < cout_k && c < cin_k) {
    const int tap = kd * 9 + kh * 3 + kw;
    v = transpose ? w[((int64_t)c * cin + m) * 27 + (26 - tap)] : w[((int64_t)m * cin + c) * 27 + tap];
  }
  wp[i] = v;
}

// LDS writes of this wavefront are done, then the workgroup meets.  (No wait on global memory: the loads of
// the rows ahead stay in flight across the barrier.)
__device__ __forceinline__ void ring_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__global__ void __launch_bounds__(256, 3) conv3d_thin_roll_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                  const float* __restrict__ bias, bf16_t* __restrict__ out,
                                                                  ThinRollArgs a) {
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63, wd = tid >> 6;
  const int W = a.in.w, H = a.in.h;
  const int G = gridDim.x;
  int t0 = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  const int tw = t0 % a.tiles_w; t0 /= a.tiles_w;
  const int seg = t0 % a.segs; t0 /= a.segs;
  const int td = t0 % a.tiles_d;
  const int n = t0 / a.tiles_d;
  const int w0 = tw * T_TW, ps0 = td * R_TD;
  const int ha = seg * a.seg_rows, hb = min(H, ha + a.seg_rows);
  const int nsteps = hb - ha + 2;         // input rows ha-1 .. hb

  bf16x8 A[12];
#pragma unroll
  for (int s = 0; s < 12; ++s) A[s] = __builtin_bit_cast(bf16x8, wp[s * 64 + lane]);

  // ---- staging role of this lane
  const int pair = wd >> 1;
  const int item = (wd & 1) * 64 + lane;
  const int grp = item % R_NG;
  const int dzs = (item / R_NG) % R_NPL, cig = item / (R_NG * R_NPL);
  const __amdgpu_buffer_rsrc_t rs_in = thin_rsrc(in + n * a.in.nstride, (uint32_t)a.in.nstride * 2);
  bool st_ok;
  int st_base;
  {
    const int p_in = ps0 - a.out.hlo + dzs - 1;       // local interior index of the input plane
    const int64_t gq = a.in.doff + p_in;
    const int sp = p_in + a.in.hlo;
    const int wc = w0 - 8 + 8 * grp;
    st_ok = item < R_ITEMS && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && wc >= 0 && wc + 8 <= W;
    st_base = 2 * (cig * 8 * (int)a.in.cstride + sp * (int)a.in.plane + wc);
  }
  const int nch = a.cin_k - cig * 8;
  const int st_dst = (cig * R_NPL + dzs) * T_P + grp - 1;
  u32x4 v[8];
  auto issue = [&](int t) {      // global loads of input row ha - 1 + t
    const int h = ha - 1 + t;
    const int vo = (st_ok && h >= 0 && h < H && t < nsteps) ? st_base + 2 * h * W : T_OOB;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      v[e] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, e < nch ? vo : T_OOB, __builtin_amdgcn_readfirstlane(2 * e * (int)a.in.cstride), 0);
  };
  auto write = [&](int slot) {   // 8 x 8 transpose into the ring
    if (item >= R_ITEMS) return;
    uint4* dst = lds + slot * R_SLOT + st_dst;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint4 u0, u1;
      u0.x = __builtin_amdgcn_perm(v[1][j], v[0][j], 0x05040100); u1.x = __builtin_amdgcn_perm(v[1][j], v[0][j], 0x07060302);
      u0.y = __builtin_amdgcn_perm(v[3][j], v[2][j], 0x05040100); u1.y = __builtin_amdgcn_perm(v[3][j], v[2][j], 0x07060302);
      u0.z = __builtin_amdgcn_perm(v[5][j], v[4][j], 0x05040100); u1.z = __builtin_amdgcn_perm(v[5][j], v[4][j], 0x07060302);
      u0.w = __builtin_amdgcn_perm(v[7][j], v[6][j], 0x05040100); u1.w = __builtin_amdgcn_perm(v[7][j], v[6][j], 0x07060302);
      const int u = 8 * grp - 6 + 2 * j;
      if (u >= 1 && u <= T_NU - 2) dst[t_pos(2 * j + 3)] = u0;
      if (u + 1 >= 1 && u + 1 <= T_NU - 2) dst[t_pos(2 * j + 4)] = u1;
    }
  };

  // ---- compute role: planes ps0 + 2 pp + {0, 1}, columns w0 + 32 cb ..
  const int pp = wd >> 1, cb = wd & 1;
  const int half = lane >> 5, col = lane & 31;
  const int ps = ps0 + 2 * pp + half;
  const int64_t gp = a.out.doff + ps - a.out.hlo;
  const bool inside = gp >= 0 && gp < a.out.dglob;          // planes outside the global volume are written as zeros
  const __amdgpu_buffer_rsrc_t rs_out = thin_rsrc(out + n * a.out.nstride, (uint32_t)a.out.nstride * 2);
  float bv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bv[i] = (bias && i < a.cout_k) ? bias[i] : 0.f;
  const int wq = w0 + cb * 32 + col;
  const int out_base = (ps < a.out.ds && wq < W) ? 2 * (ps * (int)a.out.plane + wq) : T_OOB;
  int lane_off[3];
#pragma unroll
  for (int kw = 0; kw < 3; ++kw) lane_off[kw] = (half * R_NPL + 2 * pp) * T_P + cb * 4 + t_pos(col + 2 + kw);
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;

  // ---- prologue: rows 0 and 1 into the ring, rows 2 and 3 in flight
  issue(pair);
  write(pair);
  issue(pair + 2);
  ring_barrier();

  int slot = 0;
  for (int t = 0; t < nsteps; ++t) {
    const uint4* rowbase = lds + slot * R_SLOT;
    const uint4* fp[3] = {rowbase + lane_off[0], rowbase + lane_off[1], rowbase + lane_off[2]};
    uint4 bq[3];
    bq[0] = fp[0][0];
    bq[1] = fp[1][0];
    // slide: what was accumulated under tap row kh now waits for tap row kh + 1 of the next input row
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[8 + i] = acc[4 + i];
      acc[4 + i] = acc[i];
      acc[i] = 0.f;
    }
#pragma unroll
    for (int s = 0; s < 12; ++s) {
      if (s + 2 < 12) bq[(s + 2) % 3] = fp[(s + 2) % 3][((s + 2) / 3) * T_P];
      __builtin_amdgcn_sched_barrier(0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], __builtin_bit_cast(bf16x8, bq[s % 3]), acc, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // staging turn: row t + 2 into the slot that row t - 1 has just left, then the loads of row t + 4
    if ((t & 1) == pair) {
      if (t + 2 < nsteps) write(slot == 0 ? 2 : slot - 1);
      if (t + 4 < nsteps) issue(t + 4);
    }
    if (t >= 2) {
      const int vo = out_base == T_OOB ? T_OOB : out_base + 2 * (ha + t - 2) * W;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float val = acc[8 + i] + bv[i];
        if (!(val > 0.f)) val *= a.out_slope;
        __builtin_amdgcn_raw_buffer_store_b16((short)pack_bf16x2(inside ? val : 0.f, 0.f), rs_out, i < a.cout_k ? vo : T_OOB,
                                              __builtin_amdgcn_readfirstlane(2 * i * (int)a.out.cstride), 0);
      }
    }
    ring_barrier();
    slot = slot == R_RING - 1 ? 0 : slot + 1;
  }
}

}  // namespace

bool conv3d_thin_supported(const h3d_tensor* in, const h3d_tensor* out) {
  return in->dtype == H3D_BF16 && in->c >= 1 && in->c <= 16 && out->c >= 1 && out->c <= 8 && out->w >= 32 && in->w % 2 == 0 &&
         (uintptr_t)in->data % 4 == 0;
}

// Caller guarantees conv3d_thin_supported(), 31-bit in-sample byte offsets and a 16-byte-aligned workspace
// of at least 12 KB.
h3d_status conv3d_thin(void* handle, const h3d_tensor* in, const void* w, const float* bias, h3d_tensor* out, bool transpose,
                       float out_slope, void* ws, hipStream_t stream) {
  ThinArgs a;
  a.in = make_geo(in);
  a.out = make_geo(out);
  a.cin_k = in->c; a.cout_k = out->c;
  a.out_slope = out_slope;
  a.tiles_w = (int)cdiv(out->w, T_TW);
  a.tiles_h = (int)cdiv(out->h, T_TH);
  a.tiles_d = (int)cdiv(a.out.ds, T_TD);
  const int64_t ntiles = (int64_t)out->n * a.tiles_d * a.tiles_h * a.tiles_w;
  if (ntiles == 0) return H3D_OK;
  if (ntiles >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d: too many workgroups");
  const int cin = transpose ? a.cout_k : a.cin_k, cout = transpose ? a.cin_k : a.cout_k;
  // whole 16-byte column groups: faster staging (a quarter of the load instructions)
  const bool vec8 = in->w % 8 == 0 && (uintptr_t)in->data % 16 == 0;
  if (vec8 && a.cout_k <= 4 && out->h >= 8) {
    // row streaming: pick the number of row segments that fills the chip's 3 workgroup slots per CU in the
    // fewest rounds (a segment pays for 2 extra rows and the pipeline fill)
    ThinRollArgs r;
    r.in = a.in; r.out = a.out; r.cin_k = a.cin_k; r.cout_k = a.cout_k; r.out_slope = out_slope;
    r.tiles_w = a.tiles_w;
    r.tiles_d = (int)cdiv(a.out.ds, R_TD);
    const int64_t base = (int64_t)out->n * r.tiles_d * r.tiles_w;
    const int64_t slots = 3 * (int64_t)static_cast<Handle*>(handle)->num_cu;
    int best = 1;
    int64_t best_cost = -1;
    for (int s = 1; s <= out->h / 8; ++s) {
      const int64_t cost = cdiv(base * s, slots) * (cdiv(out->h, s) + 5);
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = s; }
    }
    r.seg_rows = (int)cdiv(out->h, best);
    r.segs = (int)cdiv(out->h, r.seg_rows);
    const int64_t nwg = base * r.segs;
    if (nwg >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d: too many workgroups");
    hipLaunchKernelGGL(pack_w_thin_roll_kernel, dim3(24), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, cin, cout, transpose ? 1 : 0);
    hipLaunchKernelGGL(conv3d_thin_roll_kernel, dim3((unsigned)nwg), dim3(256), (size_t)R_RING * R_SLOT * 16, stream,
                       (const bf16_t*)in->data, (const uint4*)ws, bias, (bf16_t*)out->data, r);
    return launch_status(handle, "conv3d_thin_roll");
  }
  hipLaunchKernelGGL(pack_w_thin_kernel, dim3(18), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, cin, cout, transpose ? 1 : 0);
  constexpr size_t lds_bytes = (size_t)2 * T_CIG_UNITS * 16;
  auto kern = vec8 ? conv3d_thin_kernel<true> : conv3d_thin_kernel<false>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[vec8]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
        hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d: cannot raise the dynamic LDS limit to %zu bytes", lds_bytes);
    attr_set[vec8] = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)ntiles), dim3(T_THREADS), lds_bytes, stream, (const bf16_t*)in->data, (const uint4*)ws,
                     bias, (bf16_t*)out->data, a);
  return launch_status(handle, "conv3d_thin");
}

}  // namespace h3d
