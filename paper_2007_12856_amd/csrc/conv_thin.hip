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
// tile of rows at all: it owns 4 output planes x 64 or 128 columns and streams along H.  Per input row it keeps
// the six planes of that row in an LDS ring of three rows, computes on row t while row t+2 is being transposed
// into the ring and the global loads of the rows after it are in flight.
//   * no row halo: every input row is staged once per workgroup and its 9-tap MFMAs are issued once;
//   * with <= 4 output channels the 32 MFMA rows hold TWO output planes: row 8 kh + 4 o + m is channel m of
//     plane o under tap row kh, and the A fragment of input plane dz carries tap kd = dz - o in the rows of
//     plane o.  A wavefront = 2 planes x 64 columns: two accumulator chains of 12 MFMAs (4 input planes x 3 kw)
//     per row, and the two lane halves of an accumulator are the two planes;
//   * staging: one item per lane and row = (ci-group, plane, 8 columns): 8 loads of 16 bytes (one per channel),
//     an 8 x 8 transpose by 32 byte-permutes, eight 16-byte LDS stores.  Few, wide vector-memory instructions:
//     what the memory pipeline of a CU charges for is their number, not their bytes;
//   * for the same reason a finished output row does not leave as 2-byte stores: the wavefront transposes it
//     through 1 KB of LDS of its own and every lane stores 8 consecutive columns of one channel (16 bytes).
constexpr int R_RING = 3;
template <int TD, int CB>
struct RollCfg {
  static constexpr int TW = 32 * CB;                          // tile columns: CB MFMA column blocks, two per wavefront
  // a row of the ring: TW + 2 units (16 bytes: 8 channels of one voxel) in column order, unit x = column w0 - 1 + x:
  // the 8 consecutive lanes of a ds_read_b128 phase read 8 consecutive units, 8 distinct 16-byte bank groups.  With
  // an odd row pitch the staging stores (8 consecutive lanes = 2 neighbouring column groups x 4 rows) meet two by two.
  static constexpr int P = (TW + 2) | 1;
  static constexpr int NPL = TD + 2;
  static constexpr int SLOT = 2 * NPL * P;                    // 16-byte units of one ring slot: [ci-group][plane][unit]
  static constexpr int GROUPS = TW / 8;
  static constexpr int INNER = 2 * NPL * GROUPS;              // staging items of a row: whole column groups of the tile
  static constexpr int ITEMS = INNER + 2 * NPL * 2;           // .. and the groups left and right of it
  static constexpr int WAVES = (TD / 2) * (CB / 2);
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int OSTAGE = 72;                           // 16-byte units per wavefront: 2 planes x (32 + 4 pad)
  static constexpr size_t LDS_BYTES = ((size_t)R_RING * SLOT + WAVES * OSTAGE) * 16;
  static_assert(ITEMS <= THREADS, "one item per lane");
  static_assert(CB % 2 == 0 && TD % 2 == 0 && (2 * NPL) % 4 == 0 && GROUPS % 2 == 0, "tile shape");
};

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

template <int TD, int CB, int NSET, int WPS>
__global__ void __launch_bounds__((RollCfg<TD, CB>::THREADS), WPS) conv3d_thin_roll_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                       const float* __restrict__ bias, bf16_t* __restrict__ out,
                                                                       ThinRollArgs a) {
  using Cfg = RollCfg<TD, CB>;
  constexpr int NPL = Cfg::NPL, SLOT = Cfg::SLOT, INNER = Cfg::INNER, ITEMS = Cfg::ITEMS, GROUPS = Cfg::GROUPS, P = Cfg::P;
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63, wd = tid >> 6;
  const int W = a.in.w, H = a.in.h;
  const int G = gridDim.x;
  int t0 = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  const int tw = t0 % a.tiles_w; t0 /= a.tiles_w;
  const int seg = t0 % a.segs; t0 /= a.segs;
  const int td = t0 % a.tiles_d;
  const int n = t0 / a.tiles_d;
  const int w0 = tw * Cfg::TW, ps0 = td * TD;
  const int ha = seg * a.seg_rows, hb = min(H, ha + a.seg_rows);
  const int nsteps = hb - ha + 2;         // input rows ha-1 .. hb

  bf16x8 A[12];
#pragma unroll
  for (int s = 0; s < 12; ++s) A[s] = __builtin_bit_cast(bf16x8, wp[s * 64 + lane]);

  // ---- staging role of this lane.  The first INNER items are the column groups of the tile (8 consecutive lanes =
  // 2 neighbouring groups x 4 rows, "row" = ci-group * NPL + plane), the rest the groups left and right of it,
  // which only contribute the column next to the tile.
  const int item = tid;
  const bool inner = item < INNER;
  const bool edge = !inner && item < ITEMS;
  const bool left = item - INNER < 2 * NPL;
  int grp, rowid;
  if (inner) {
    const int q = item >> 3;                         // (row group of 4, pair of column groups)
    grp = 2 * (q % (GROUPS / 2)) + (item & 1);
    rowid = 4 * (q / (GROUPS / 2)) + ((item >> 1) & 3);
  } else {
    grp = left ? -1 : GROUPS;
    rowid = (item - INNER) % (2 * NPL);
  }
  const int dzs = rowid % NPL, cig = rowid / NPL;
  const __amdgpu_buffer_rsrc_t rs_in = thin_rsrc(in + n * a.in.nstride, (uint32_t)a.in.nstride * 2);
  bool st_ok;
  int st_base;
  {
    const int p_in = ps0 - a.out.hlo + dzs - 1;       // local interior index of the input plane
    const int64_t gq = a.in.doff + p_in;
    const int sp = p_in + a.in.hlo;
    const int wc = w0 + 8 * grp;
    st_ok = item < ITEMS && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && wc >= 0 && wc + 8 <= W;
    st_base = 2 * (cig * 8 * (int)a.in.cstride + sp * (int)a.in.plane + wc);
  }
  const int nch = a.cin_k - cig * 8;
  // column w0 + 8 grp + c is unit 8 grp + 1 + c of its row; the left group's last column is unit 0, the right group's
  // first column unit TW + 1
  const int st_p0 = rowid * P + (inner ? 8 * grp + 1 : (left ? 0 : Cfg::TW + 1));
  auto issue = [&](u32x4 (&v)[8], int t) {      // global loads of input row ha - 1 + t
    const int h = ha - 1 + t;
    const int vo = (st_ok && h >= 0 && h < H && t < nsteps) ? st_base + 2 * h * W : T_OOB;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      v[e] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, e < nch ? vo : T_OOB, __builtin_amdgcn_readfirstlane(2 * e * (int)a.in.cstride), 0);
  };
  auto write = [&](const u32x4 (&v)[8], int slot) {   // 8 x 8 transpose into the ring
    uint4* dst = lds + slot * SLOT + st_p0;
    if (inner) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {       // dword j of each channel = columns 2j, 2j+1 of the group
        uint4 u0, u1;
        u0.x = __builtin_amdgcn_perm(v[1][j], v[0][j], 0x05040100); u1.x = __builtin_amdgcn_perm(v[1][j], v[0][j], 0x07060302);
        u0.y = __builtin_amdgcn_perm(v[3][j], v[2][j], 0x05040100); u1.y = __builtin_amdgcn_perm(v[3][j], v[2][j], 0x07060302);
        u0.z = __builtin_amdgcn_perm(v[5][j], v[4][j], 0x05040100); u1.z = __builtin_amdgcn_perm(v[5][j], v[4][j], 0x07060302);
        u0.w = __builtin_amdgcn_perm(v[7][j], v[6][j], 0x05040100); u1.w = __builtin_amdgcn_perm(v[7][j], v[6][j], 0x07060302);
        dst[2 * j] = u0;
        dst[2 * j + 1] = u1;
      }
    } else if (edge) {
      // left group: its last column (high half of dword 3) is unit 0; right group: its first column is unit TW + 1
      const uint32_t sel = left ? 0x07060302 : 0x05040100;
      uint4 u;
      u.x = __builtin_amdgcn_perm(left ? v[1][3] : v[1][0], left ? v[0][3] : v[0][0], sel);
      u.y = __builtin_amdgcn_perm(left ? v[3][3] : v[3][0], left ? v[2][3] : v[2][0], sel);
      u.z = __builtin_amdgcn_perm(left ? v[5][3] : v[5][0], left ? v[4][3] : v[4][0], sel);
      u.w = __builtin_amdgcn_perm(left ? v[7][3] : v[7][0], left ? v[6][3] : v[6][0], sel);
      dst[0] = u;
    }
  };

  // ---- compute role: planes ps0 + 2 pp + {0, 1}, columns w0 + 64 cp .. + 63 (column blocks 2 cp and 2 cp + 1)
  const int pp = wd / (CB / 2), cp = wd % (CB / 2);
  const int half = lane >> 5, col = lane & 31;
  float bv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bv[i] = (bias && i < a.cout_k) ? bias[i] : 0.f;
  const bool inside = [&] {          // planes outside the global volume are written as zeros
    const int64_t gp = a.out.doff + (ps0 + 2 * pp + half) - a.out.hlo;
    return gp >= 0 && gp < a.out.dglob;
  }();
  // output transpose: [plane o][channel i][64 columns] bf16, planes 36 units apart; lane j then owns the unit
  // (o, i, column group g) = 8 consecutive columns of one channel
  bf16_t* ost_w = reinterpret_cast<bf16_t*>(lds + R_RING * SLOT + wd * Cfg::OSTAGE + half * 36) + col;
  const uint4* ost_r = lds + R_RING * SLOT + wd * Cfg::OSTAGE + (lane >> 5) * 36 + (lane & 31);
  const __amdgpu_buffer_rsrc_t rs_out = thin_rsrc(out + n * a.out.nstride, (uint32_t)a.out.nstride * 2);
  int out_base;
  {
    const int o = lane >> 5, i = (lane >> 3) & 3, g = lane & 7;
    const int ps = ps0 + 2 * pp + o, wq = w0 + 64 * cp + 8 * g;
    out_base = (ps < a.out.ds && wq < W && i < a.cout_k) ? 2 * (i * (int)a.out.cstride + ps * (int)a.out.plane + wq) : T_OOB;
  }
  const int lane_off = (half * NPL + 2 * pp) * P + cp * 64 + col;      // unit of column w0 + 64 cp + col - 1 (tap kw = 0)
  f32x16 acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

  // ---- prologue: rows 0 and 1 into the ring, rows 2 .. 1 + NSET in flight (row r waits in register set r % NSET)
  u32x4 v[NSET][8];
  {
    u32x4 v1[8];
    issue(v[0], 0);
    issue(v1, 1);
    write(v[0], 0);
    write(v1, 1);
  }
#pragma unroll
  for (int r = 2; r < 2 + NSET; ++r) issue(v[r % NSET], r);
  ring_barrier();

  // B fragments are read R_AHEAD (dz, kw) steps ahead, across the row boundary: row t + 1 is complete in its slot
  // before row t's barrier (it was written during row t - 1), so the queue never drains between rows
  constexpr int R_AHEAD = 3;
  static_assert(12 % R_AHEAD == 0, "fragment s lives in queue entry s % R_AHEAD in every row");
  const uint4* fp = lds + lane_off;
  uint4 bq[R_AHEAD][2];
#pragma unroll
  for (int s = 0; s < R_AHEAD; ++s)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) bq[s][cb] = fp[(s / 3) * P + s % 3 + 32 * cb];

  int slot = 0;
  for (int t0s = 0; t0s < nsteps; t0s += NSET) {
#pragma unroll
  for (int k = 0; k < NSET; ++k) {
    const int t = t0s + k;
    if (t >= nsteps) break;
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
    for (int s = 0; s < 12; ++s) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], __builtin_bit_cast(bf16x8, bq[s % R_AHEAD][cb]), acc[cb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (s + R_AHEAD == 12) fp += (slot == R_RING - 1 ? -(R_RING - 1) : 1) * SLOT;      // the queue moves on to the next row's slot
      const int f = (s + R_AHEAD) % 12;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) bq[s % R_AHEAD][cb] = fp[(f / 3) * P + f % 3 + 32 * cb];
    }
    __builtin_amdgcn_sched_barrier(0);
    // row t + 2 goes into the slot that row t - 1 has just left; then the loads of row t + 2 + NSET
    if (t + 2 < nsteps) write(v[(k + 2) % NSET], slot == 0 ? 2 : slot - 1);
    if (t + 2 + NSET < nsteps) issue(v[(k + 2) % NSET], t + 2 + NSET);
    if (t >= 2) {
      // finished output row ha + t - 2: bias, activation, bf16, transposed through this wavefront's LDS patch
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float val = acc[cb][8 + i] + bv[i];
          if (!(val > 0.f)) val *= a.out_slope;
          ost_w[i * 64 + cb * 32] = (bf16_t)pack_bf16x2(inside ? val : 0.f, 0.f);
        }
      asm volatile("" ::: "memory");     // the 16-byte read below aliases the 2-byte writes above
      const uint4 o4 = *ost_r;
      const int vo = out_base == T_OOB ? T_OOB : out_base + 2 * (ha + t - 2) * W;
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o4), rs_out, vo, 0, 0);
    }
    ring_barrier();
    slot = slot == R_RING - 1 ? 0 : slot + 1;
  }
  }
}

template <int TD, int CB, int NSET, int WPS>
h3d_status launch_thin_roll(void* handle, const h3d_tensor* in, const float* bias, h3d_tensor* out, const ThinArgs& a, float out_slope,
                            const void* wp, hipStream_t stream) {
  using Cfg = RollCfg<TD, CB>;
  auto kern = conv3d_thin_roll_kernel<TD, CB, NSET, WPS>;
  static int wgs_per_cu = 0;
  if (wgs_per_cu == 0) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES) !=
        hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d: cannot raise the dynamic LDS limit to %zu bytes", Cfg::LDS_BYTES);
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, Cfg::THREADS, Cfg::LDS_BYTES) != hipSuccess || nb < 1) nb = 1;
    wgs_per_cu = nb;
  }
  ThinRollArgs r;
  r.in = a.in; r.out = a.out; r.cin_k = a.cin_k; r.cout_k = a.cout_k; r.out_slope = out_slope;
  r.tiles_w = (int)cdiv(out->w, Cfg::TW);
  r.tiles_d = (int)cdiv(a.out.ds, TD);
  // pick the number of row segments that fills the chip's workgroup slots in the fewest rounds (a segment pays for
  // 2 extra rows and the pipeline fill)
  const int64_t base = (int64_t)out->n * r.tiles_d * r.tiles_w;
  const int64_t slots = (int64_t)wgs_per_cu * static_cast<Handle*>(handle)->num_cu;
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
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(Cfg::THREADS), Cfg::LDS_BYTES, stream, (const bf16_t*)in->data, (const uint4*)wp, bias,
                     (bf16_t*)out->data, r);
  return launch_status(handle, "conv3d_thin_roll");
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
  if (vec8 && a.cout_k <= 4 && out->h >= 8 && (uintptr_t)out->data % 16 == 0) {
    hipLaunchKernelGGL(pack_w_thin_roll_kernel, dim3(24), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, cin, cout, transpose ? 1 : 0);
    // wide rows: 128-column tiles (a 64-column tile also pulls in the neighbouring 128-byte line of every row for
    // the one column next to it)
    if (out->w > 64) return launch_thin_roll<4, 4, 1, 2>(handle, in, bias, out, a, out_slope, ws, stream);
    return launch_thin_roll<4, 2, 1, 2>(handle, in, bias, out, a, out_slope, ws, stream);
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
