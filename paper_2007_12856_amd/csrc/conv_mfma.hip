// bf16 MFMA implicit-GEMM kernels for the 3x3x3 convolution passes on gfx950.
//
// Forward / backward-data (one kernel; backward-data is the forward correlation of
// g = dz * act'(z) with the weights transposed and reversed, Sec. III-C "BD"):
//   D[co][voxel] = sum_{tap, ci} Wp[co][tap, ci] * X[tap, ci][voxel]
//   * output channels sit on the MFMA rows (A operand = weights), voxels on the columns
//     (B operand = input patches), so one accumulator register of a wavefront covers 32
//     consecutive W positions of one channel: stores along W are contiguous;
//   * the contraction index is ordered (tap, ci) with ci fastest: the 8 bf16 a lane feeds to
//     v_mfma_f32_32x32x16_bf16 are 8 consecutive input channels of ONE voxel.  NCDHW keeps
//     channels a whole volume apart, so the input tile (with its halo) is transposed on its way
//     into LDS: 16-byte units of 8 channels, laid out [ci-group][d][h][w], read back with
//     conflict-free ds_read_b128 at the 27 shifted offsets;
//   * weights are pre-packed in exact fragment order ([co-block][ci-chunk][tap][lane][8]) and go
//     global -> registers (fully coalesced 1 KB per fragment, L1/L2 resident), prefetched one
//     (kd,kw) step ahead; they never touch LDS;
//   * a workgroup is 8 wavefronts: NCB blocks of 32 output channels x ND depth planes; each
//     wavefront owns 32 channels x 128 voxels (4 MFMA column blocks = 4 groups of h rows).  For a
//     fixed (kd,kw) the 12 (block, kh) products need only 3*RPB+3 distinct row fragments, so LDS
//     read traffic is about half of one fragment per MFMA;
//   * the ci loop runs in chunks of 16 channels with two LDS buffers: the global loads of chunk
//     c+1 are in flight while chunk c is multiplied.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int CI_CHUNK = 16;
constexpr int WG_THREADS = 512;

// wp: [co_blk][chunk][tap][lane][8] bf16; lane l, element e: co_k = 32*co_blk + l%32, ci_k = 16*chunk + 8*(l/32) + e
__global__ void pack_w_mfma_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout, int transpose,
                                   int nchunks, int ncoblk) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t total = (int64_t)ncoblk * nchunks * 27 * 512;
  if (i >= total) return;
  int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  int64_t r = i >> 9;
  int tap = (int)(r % 27); r /= 27;
  int chunk = (int)(r % nchunks);
  int cb = (int)(r / nchunks);
  int co_k = cb * 32 + (lane & 31), ci_k = chunk * CI_CHUNK + (lane >> 5) * 8 + e;
  int cin_k = transpose ? cout : cin, cout_k = transpose ? cin : cout;
  bf16_t v = 0;
  if (co_k < cout_k && ci_k < cin_k)
    v = transpose ? w[((int64_t)ci_k * cin + co_k) * 27 + (26 - tap)] : w[((int64_t)co_k * cin + ci_k) * 27 + tap];
  wp[i] = v;
}

struct MfmaArgs {
  Geo in, mask, out;
  int cin_k, cout_k, nchunks, ncoblk;
  int tiles_w, tiles_h, tiles_d, ntiles;
  float out_slope, mask_slope;
  // split of the input-channel chunks over blockIdx.z (small volumes with many channels would otherwise
  // occupy a handful of CUs): each split writes fp32 partial sums, a second kernel adds them in order
  int csplit, chunks_per_split;
  float* part;      // [csplit][n][cout][stored planes][h][w], used when csplit > 1
};

__device__ __forceinline__ uint32_t mask_pair(uint32_t v, uint32_t m, float slope) {
  // per bf16 half: keep v where the mask value is > 0, else v * slope (rounded to bf16)
  float v0 = __uint_as_float(v << 16), v1 = __uint_as_float(v & 0xffff0000u);
  float m0 = __uint_as_float(m << 16), m1 = __uint_as_float(m & 0xffff0000u);
  if (!(m0 > 0.f)) v0 *= slope;
  if (!(m1 > 0.f)) v1 *= slope;
  return (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int BUF_OOB = (int)0x80000000;   // byte offset beyond every buffer: such a lane reads zero

// The descriptor must live in scalar registers: the pointer is passed through readfirstlane so the
// compiler knows it is wave-uniform (otherwise every load becomes a waterfall loop).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  void* q = reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(q, 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

// VEC: rows start 4-byte aligned and W is even, so a pair of bf16 is one dword load (the normal case);
// otherwise the two elements of a pair are fetched by two 2-byte loads with their own validity.
// FLAT: for outputs of one or two planes (the halo strips of a main / halo split) the ND wavefronts of a
// channel block take ND groups of rows of ONE plane instead of ND planes, so no wavefront runs empty.
template <int NCB, int ND, int TWC, bool MASKED, bool VEC, bool SPLIT, bool FLAT>
__global__ void __launch_bounds__(WG_THREADS) conv3d_mfma_kernel(const bf16_t* __restrict__ in, const bf16_t* __restrict__ mask,
                                                                 const uint4* __restrict__ wp, const float* __restrict__ bias,
                                                                 bf16_t* __restrict__ out, MfmaArgs a) {
  static_assert(NCB * ND == 8, "8 wavefronts per workgroup");
  constexpr int RPB = 32 / TWC;        // h rows per MFMA column block
  constexpr int TH = 4 * RPB, TW = TWC;   // rows per wavefront
  constexpr int TDP = FLAT ? 1 : ND, THT = FLAT ? TH * ND : TH;   // planes and rows of the workgroup's tile
  constexpr int TD2 = TDP + 2, TH2 = THT + 2;
  constexpr int P = TWC == 32 ? 36 : 20;   // LDS row pitch in 16-byte units: w in [w0-2, w0+TW+2)
  constexpr int PAIRS = (TW + 4) / 2;
  constexpr int CIG_UNITS = TD2 * TH2 * P;
  constexpr int BUF_UNITS = 2 * CIG_UNITS;
  constexpr int NITEMS = 2 * TD2 * TH2 * PAIRS;
  constexpr int ROUNDS = (NITEMS + WG_THREADS - 1) / WG_THREADS;
  constexpr int NFRAG = 3 * RPB + 3;   // distinct start rows b*RPB + kh
  extern __shared__ uint4 lds[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cbw = wave / ND, wd = wave % ND;
  const int co_blk = blockIdx.y * NCB + cbw;
  const int W = a.in.w, H = a.in.h;

  // ---- tile-invariant part of the staging plan: which units this thread fills
  int lds_unit[ROUNDS], item_meta[ROUNDS];   // meta: pair | hy << 8 | dz << 16 | cig << 24 (cig 2: no item)
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    int item = tid + r * WG_THREADS;
    int pair = item % PAIRS;
    int x = item / PAIRS;
    int hy = x % TH2; x /= TH2;
    int dz = x % TD2;
    int cig = item < NITEMS ? x / TD2 : 2;
    lds_unit[r] = (cig * TD2 + dz) * (TH2 * P) + hy * P + 2 * pair;
    item_meta[r] = pair | (hy << 8) | (dz << 16) | (cig << 24);
  }

  // ---- per-tile part: byte offsets of this thread's items inside the sample (ci-group included),
  //      BUF_OOB where the item lies outside the volume: a buffer load then returns zero without
  //      any branch or select.  The channel inside the chunk is added as a scalar offset.
  constexpr int NV = VEC ? 1 : 2;
  int voff[ROUNDS][NV], moffb[MASKED ? ROUNDS : 1][NV];
  int n_plan = 0;   // sample index of the planned tile (wave-uniform)
  const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(wp, (uint32_t)a.ncoblk * a.nchunks * 27 * 1024);
  auto plan_tile = [&](int tile) {
    int t = tile;
    const int tw = t % a.tiles_w; t /= a.tiles_w;
    const int th = t % a.tiles_h; t /= a.tiles_h;
    const int td = t % a.tiles_d;
    const int n = t / a.tiles_d;
    const int w0 = tw * TW, h0 = th * THT, ps0 = td * TDP;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int m = item_meta[r];
      const int pair = m & 0xff, hy = (m >> 8) & 0xff, dz = (m >> 16) & 0xff, cig = m >> 24;
      const int p_in = ps0 - a.out.hlo + dz - 1;        // local interior index of the input plane
      const int64_t gq = a.in.doff + p_in;
      const int sp = p_in + a.in.hlo;
      const int h = h0 + hy - 1, w = w0 - 2 + 2 * pair;
      const bool ok = cig < 2 && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H;
      const int base = 2 * (cig * 8 * (int)a.in.cstride + sp * (int)a.in.plane + h * W + w);
      const int mbase = MASKED ? 2 * (cig * 8 * (int)a.mask.cstride + (p_in + a.mask.hlo) * (int)a.mask.plane + h * W + w) : 0;
#pragma unroll
      for (int e2 = 0; e2 < NV; ++e2) {
        const bool okw = VEC ? (ok && w >= 0 && w + 1 < W) : (ok && w + e2 >= 0 && w + e2 < W);
        voff[r][e2] = okw ? base + 2 * e2 : BUF_OOB;
        if (MASKED) moffb[r][e2] = okw ? mbase + 2 * e2 : BUF_OOB;
      }
    }
    n_plan = n;
  };

  uint32_t v[ROUNDS][8];
  uint32_t mv[MASKED ? ROUNDS : 1][8];

  // `live` = false turns every load into an out-of-range (zero, no traffic) one: the last stage of a
  // workgroup has nothing to prefetch, but keeping the load count identical on every path lets the
  // compiler use exact s_waitcnt counts for the weight fragments instead of waiting for everything.
  auto load_chunk = [&](int c, bool live) {
    const bool full = (c + 1) * CI_CHUNK <= a.cin_k;   // uniform: no channel of this chunk is beyond Cin
    const __amdgpu_buffer_rsrc_t rs_in = make_rsrc(in + n_plan * a.in.nstride, (uint32_t)a.in.nstride * 2);
    const __amdgpu_buffer_rsrc_t rs_mask = make_rsrc(MASKED ? mask + n_plan * a.mask.nstride : in, (uint32_t)a.mask.nstride * 2);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int soff = __builtin_amdgcn_readfirstlane(2 * (c * CI_CHUNK + e) * (int)a.in.cstride);
      const int smoff = MASKED ? __builtin_amdgcn_readfirstlane(2 * (c * CI_CHUNK + e) * (int)a.mask.cstride) : 0;
#pragma unroll
      for (int r = 0; r < ROUNDS; ++r) {
        int vo[NV], mo[NV];
#pragma unroll
        for (int e2 = 0; e2 < NV; ++e2) {
          vo[e2] = live ? voff[r][e2] : BUF_OOB;
          mo[e2] = MASKED ? (live ? moffb[r][e2] : BUF_OOB) : 0;
          if (!full) {
            const bool chan_ok = c * CI_CHUNK + (item_meta[r] >> 24) * 8 + e < a.cin_k;
            vo[e2] = chan_ok ? vo[e2] : BUF_OOB;
            mo[e2] = chan_ok ? mo[e2] : BUF_OOB;
          }
        }
        if (VEC) {
          v[r][e] = __builtin_amdgcn_raw_buffer_load_b32(rs_in, vo[0], soff, 0);
          if (MASKED) mv[r][e] = __builtin_amdgcn_raw_buffer_load_b32(rs_mask, mo[0], smoff, 0);
        } else {
          const uint32_t lo = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_in, vo[0], soff, 0);
          const uint32_t hi = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_in, vo[NV - 1], soff, 0);
          v[r][e] = lo | (hi << 16);
          if (MASKED) {
            const uint32_t ml = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_mask, mo[0], smoff, 0);
            const uint32_t mh = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_mask, mo[NV - 1], smoff, 0);
            mv[r][e] = ml | (mh << 16);
          }
        }
      }
    }
  };

  auto store_chunk = [&](int buf) {
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      if ((item_meta[r] >> 24) >= 2) continue;
      uint32_t g[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) g[e] = MASKED ? mask_pair(v[r][e], mv[r][e], a.mask_slope) : v[r][e];
      uint4 u0, u1;   // unit of w (low halves) and of w+1 (high halves): 8 channels each
      u0.x = __builtin_amdgcn_perm(g[1], g[0], 0x05040100); u1.x = __builtin_amdgcn_perm(g[1], g[0], 0x07060302);
      u0.y = __builtin_amdgcn_perm(g[3], g[2], 0x05040100); u1.y = __builtin_amdgcn_perm(g[3], g[2], 0x07060302);
      u0.z = __builtin_amdgcn_perm(g[5], g[4], 0x05040100); u1.z = __builtin_amdgcn_perm(g[5], g[4], 0x07060302);
      u0.w = __builtin_amdgcn_perm(g[7], g[6], 0x05040100); u1.w = __builtin_amdgcn_perm(g[7], g[6], 0x07060302);
      uint4* dst = lds + buf * BUF_UNITS + lds_unit[r];
      dst[0] = u0;
      dst[1] = u1;
    }
  };

  const bool wave_active = co_blk < a.ncoblk;
  const int j = lane & 31;
  // accumulators start from the bias of their output channel (row 8*(r/4) + 4*(lane/32) + r%4 of the block)
  f32x16 acc[4];
  auto init_acc = [&]() {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = co_blk * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
      const float bv = (bias && co < a.cout_k) ? bias[co] : 0.f;
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[b][r] = bv;
    }
  };
  init_acc();

  const int lane_unit = (lane >> 5) * CIG_UNITS + ((FLAT ? 0 : wd) * TH2 + (FLAT ? wd * TH : 0) + j / TWC) * P + (j % TWC) + 1;

  const int a_voff = ((wave_active ? co_blk : 0) * a.nchunks * 27 * 64 + lane) * 16;
  auto load_a = [&](int c, int step, uint4 (&dst)[3]) {
    const int kd = step / 3, kw = step % 3;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
      const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rs_w, a_voff, __builtin_amdgcn_readfirstlane((c * 27 + kd * 9 + kh * 3 + kw) * 1024), 0);
      dst[kh] = uint4{t.x, t.y, t.z, t.w};
    }
  };

  // One chunk = 9 (kd,kw) steps of 12 MFMAs.  Vector-memory loads return in order, so a wait for a
  // weight fragment also waits for every load issued before it.  The weight fragments of the first
  // APRE steps are therefore requested BEFORE the (long-latency) input loads of the next stage are
  // issued (`issue_next`), and the remaining ones only once those have had several steps to land.
  constexpr int APRE = 5;
  auto compute_chunk = [&](int c, int buf, auto&& issue_next) {
    const uint4* base = lds + buf * BUF_UNITS + lane_unit;
    uint4 afr[9][3];
    uint4 bfr[2][NFRAG];     // row fragments of the current and of the next (kd,kw) step
    auto load_b = [&](int step, uint4 (&dst)[NFRAG]) {
      const int kd = step / 3, kw = step % 3;
#pragma unroll
      for (int s = 0; s < NFRAG; ++s) dst[s] = base[(kd * TH2 + s) * P + kw];
    };
#pragma unroll
    for (int step = 0; step < APRE; ++step) load_a(c, step, afr[step]);
    load_b(0, bfr[0]);
    __builtin_amdgcn_sched_barrier(0);   // keep the weight requests ahead of the input loads ...
    issue_next();
    __builtin_amdgcn_sched_barrier(0);   // ... and the input loads ahead of the MFMA steps (not sunk below them)
#pragma unroll
    for (int step = 0; step < 9; ++step) {
      if (step + 1 < 9) load_b(step + 1, bfr[(step + 1) & 1]);     // in flight during this step's MFMAs
      if (step == APRE - 1) {
#pragma unroll
        for (int s2 = APRE; s2 < 9; ++s2) load_a(c, s2, afr[s2]);
      }
#pragma unroll
      for (int s = 0; s < NFRAG; ++s) {
        const bf16x8 B = __builtin_bit_cast(bf16x8, bfr[step & 1][s]);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
          // the block whose start row b*RPB + kh equals s
          if (s - kh >= 0 && (s - kh) % RPB == 0 && (s - kh) / RPB < 4) {
            const int b = (s - kh) / RPB;
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afr[step][kh]), B, acc[b], 0, 0, 0);
          }
        }
      }
    }
  };

  // activation, bf16 store (the bias is already in the accumulators); output planes outside the global
  // volume are zero.  Buffer stores: the lane's voxel offset (BUF_OOB where the voxel is beyond H or W:
  // such a store is dropped) plus a scalar channel offset — no branches, no 64-bit address arithmetic.
  auto epilogue = [&](int tile) {
    int t = tile;
    const int tw = t % a.tiles_w; t /= a.tiles_w;
    const int th = t % a.tiles_h; t /= a.tiles_h;
    const int td = t % a.tiles_d;
    const int n = t / a.tiles_d;
    const int w0 = tw * TW, h0 = th * THT + (FLAT ? wd * TH : 0), ps = td * TDP + (FLAT ? 0 : wd);
    if (!wave_active || ps >= a.out.ds) return;
    const int64_t gp = a.out.doff + ps - a.out.hlo;
    const bool inside = gp >= 0 && gp < a.out.dglob;
    const int row_ch = 4 * (lane >> 5);   // this lane's accumulator rows are channels 8*(r/4) + row_ch + r%4 of the block
    if (SPLIT) {
      // the accumulators go out as they are, [split][tile][channel block][plane of the tile][b*16 + r][lane]: every
      // store instruction writes 256 contiguous bytes; the reduction kernel undoes the mapping
      float* pp = a.part + (((((int64_t)blockIdx.z * a.ntiles + tile) * a.ncoblk + co_blk) * ND + wd) * 64) * 64 + lane;
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) pp[(b * 16 + r) * 64] = acc[b][r];
      return;
    }
    const __amdgpu_buffer_rsrc_t rs_out = make_rsrc(out + n * a.out.nstride, (uint32_t)a.out.nstride * 2);
    if (VEC) {
      // Two adjacent voxels live in adjacent lanes.  Lane pairs swap one value (DPP quad_perm [1,0,3,2])
      // so that the even lane holds both voxels of channel row r and the odd lane both voxels of row
      // r+1: every lane then stores ONE dword (two bf16) instead of two shorts.
      const bool odd = lane & 1;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int h = h0 + b * RPB + j / TWC, w = w0 + (j % TWC) - (odd ? 1 : 0);
        const int vo = (h < H && w < W)
                           ? 2 * ((row_ch + (odd ? 1 : 0)) * (int)a.out.cstride + ps * (int)a.out.plane + h * W + w) : BUF_OOB;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const int co_u = co_blk * 32 + 8 * (r / 4) + (r % 4);          // wave-uniform part of the even lane's channel
          const bool ch_ok = co_u + row_ch + (odd ? 1 : 0) < a.cout_k;
          float v0 = acc[b][r], v1 = acc[b][r + 1];
          if (!(v0 > 0.f)) v0 *= a.out_slope;
          if (!(v1 > 0.f)) v1 *= a.out_slope;
          const float give = odd ? v0 : v1;
          const float got = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(give), 0xB1, 0xF, 0xF, true));
          const uint32_t pk = odd ? pack_bf16x2(got, v1) : pack_bf16x2(v0, got);
          __builtin_amdgcn_raw_buffer_store_b32(inside ? pk : 0u, rs_out, ch_ok ? vo : BUF_OOB,
                                                __builtin_amdgcn_readfirstlane(2 * co_u * (int)a.out.cstride), 0);
        }
      }
    } else {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int h = h0 + b * RPB + j / TWC, w = w0 + j % TWC;
        const int vo = (h < H && w < W) ? 2 * (row_ch * (int)a.out.cstride + ps * (int)a.out.plane + h * W + w) : BUF_OOB;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co_u = co_blk * 32 + 8 * (r / 4) + (r % 4);            // wave-uniform part of the channel
          const bool ch_ok = co_u + row_ch < a.cout_k;
          float val = acc[b][r];
          if (!(val > 0.f)) val *= a.out_slope;
          __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16(inside ? val : 0.f), rs_out, ch_ok ? vo : BUF_OOB,
                                                __builtin_amdgcn_readfirstlane(2 * co_u * (int)a.out.cstride), 0);
        }
      }
    }
  };

  // ---- persistent loop: this workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ...; the
  //      (tile, ci-chunk) stages alternate between two LDS buffers, and the global loads of the next
  //      stage — the next chunk, or chunk 0 of the NEXT TILE — are in flight while this one is multiplied
  // consecutive workgroup ids land on different XCDs (each with its own L2): remap so that the
  // workgroups of one XCD work on neighbouring tiles and share the halo lines in that L2
  const int G = gridDim.x;
  int tile = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  if (tile >= a.ntiles) return;
  const int c_begin = SPLIT ? blockIdx.z * a.chunks_per_split : 0;
  const int c_end = SPLIT ? min(a.nchunks, c_begin + a.chunks_per_split) : a.nchunks;
  plan_tile(tile);
  load_chunk(c_begin, true);
  store_chunk(0);
  __syncthreads();
  int buf = 0;
  while (true) {
    for (int c = c_begin; c < c_end; ++c) {
      const bool last_chunk = c + 1 == c_end;
      const int next_tile = tile + G;
      const bool more = !last_chunk || next_tile < a.ntiles;
      auto issue_next = [&]() {
        if (last_chunk && more) plan_tile(next_tile);
        load_chunk(last_chunk ? c_begin : c + 1, more);
      };
      if (wave_active) compute_chunk(c, buf, issue_next);
      else issue_next();
      if (more) store_chunk(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
    epilogue(tile);
    init_acc();
    tile += G;
    if (tile >= a.ntiles) break;
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Wide-blocked form of the same implicit GEMM for the large layers (more than 16 columns, at least 3 stored output
// planes, no fused mask): FOUR wavefronts per workgroup, one per SIMD, each owning CB blocks of 32 output channels x
// 8 MFMA column blocks (8 rows x 32 columns of one plane = 256 voxels): CB * 8 accumulator tiles = up to 256
// registers, which the compiler keeps in the accumulation registers.  Per (kd,kw) step a wavefront then needs 3 * CB
// weight fragments and 10 row fragments for 24 * CB products: one weight fragment feeds 8 products and one row
// fragment up to 3 * CB, against 4 and 2-3 in the kernel above, so the weight stream from L2 and the LDS reads per
// product are both halved, and a chunk of 16 input channels is 216 * CB products per wavefront between two barriers.
// With one wavefront per SIMD nothing hides a stall, so everything is requested ahead: weight fragments one step
// ahead (two register sets; they do not depend on the tile, so the stream runs on across chunk and tile borders),
// row fragments one step ahead (a register is refilled as soon as its last product has been issued), and the input
// of the next stage in two groups of 8 channels (40 registers) that are requested in thirds at steps 0-2 and 4-6 and
// written to the other LDS buffer at step 4 and after step 8.  Vector-memory operations return in issue order and
// share one counter, so a wait for the weight fragments of step s + 1 also waits for the input requests issued
// before them, i.e. up to step s - 1: the input stream has about two steps (3000 cycles) of latency to hide in, not
// half a chunk; a third weight set would add a step but does not fit the 512 registers.
// Measured by switching parts off (128 -> 64 channels on 64 x 256 x 256, one box): with the output stores redirected
// into a 64 KB window that stays in the L2 the kernel takes 1.19 instead of 1.44 ms although it issues the same
// instructions - 5 % fewer cycles and a shader clock of 2.14 instead of 1.85 GHz; cache-policy bits on the stores and a
// staggered start of the workgroups change nothing.  The 537 MB of output cost about 0.25 ms that nothing in the kernel
// hides.
// The sums are taken in the order of the kernel above (chunk, kd, kw, kh), so the two give identical bits.
// WCB = 2 (the form that runs for more than 32 output channels, with CB = 1): EIGHT wavefronts per workgroup, two per
// SIMD and plane, each with its own channel block of the same tile: a wavefront holds 128 accumulators and 256
// registers in all, the staged input serves the same 64 channels as with CB = 2, and while one wavefront of a SIMD waits
// (request, LDS, barrier, epilogue stores) the other multiplies.  Measured against the four-wavefront CB = 2 form on one
// box, seven layers of the U-Net level: 4 to 9 % faster on every one (128->64: 1.48 -> 1.43 ms, 32->64: 0.505 -> 0.46).
// Instantiated: <1, 1> and <1, 1, 2> (at most 32 output channels, or small volumes) and <1, 2>.
// RSP = 2 (for layers with a single block of output channels): eight wavefronts as well, the two of a plane taking
// four rows of the tile each (64 accumulators, 6 row fragments per step).
template <int CB, int WCB, int RSP = 1>
__global__ void __launch_bounds__(256 * WCB * RSP) conv3d_mfma_wide_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wp,
                                                                     const float* __restrict__ bias, bf16_t* __restrict__ out, MfmaArgs a) {
  static_assert(WCB * RSP <= 2, "at most eight wavefronts");
  constexpr int NT = 256 * WCB * RSP;
  constexpr int TD = 4, TH = 8, TW = 32, VB = TH / RSP;      // VB: row blocks (of 32 voxels) per wavefront
  constexpr int TD2 = TD + 2, TH2 = TH + 2;
  constexpr int P = 36, PAIRS = 18;            // LDS row: w in [w0-2, w0+34), 16-byte units of 8 channels
  constexpr int CIG_UNITS = TD2 * TH2 * P;
  constexpr int BUF_UNITS = 2 * CIG_UNITS;
  constexpr int NITEMS = TD2 * TH2 * PAIRS;   // (plane, row, pair of columns) items of one channel group
  constexpr int ROUNDS = (NITEMS + NT - 1) / NT;
  constexpr int NFRAG = VB + 2;
  extern __shared__ uint4 lds[];

  const int tid = threadIdx.x, lane = tid & 63, wd = (tid >> 6) & 3;      // plane of the tile
  const int wcb = WCB == 2 ? tid >> 8 : 0, rh = RSP == 2 ? tid >> 8 : 0;   // channel-block group, row half
  const int co_blk0 = (blockIdx.y * WCB + wcb) * CB;
  const int W = a.in.w, H = a.in.h;

  int lds_unit[ROUNDS], item_meta[ROUNDS];     // meta: pair | hy << 8 | dz << 16 | valid << 24
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int item = tid + r * NT;
    const int pair = item % PAIRS;
    int x = item / PAIRS;
    const int hy = x % TH2; x /= TH2;
    const int dz = x % TD2;
    const int valid = item < NITEMS ? 1 : 0;
    lds_unit[r] = (dz * TH2 + hy) * P + 2 * pair;
    item_meta[r] = pair | (hy << 8) | (dz << 16) | (valid << 24);
  }

  int voff[ROUNDS];
  int n_plan = 0;
  const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(wp, (uint32_t)a.ncoblk * a.nchunks * 27 * 1024);
  auto plan_tile = [&](int tile) {
    int t = tile;
    const int tw = t % a.tiles_w; t /= a.tiles_w;
    const int th = t % a.tiles_h; t /= a.tiles_h;
    const int td = t % a.tiles_d;
    const int n = t / a.tiles_d;
    const int w0 = tw * TW, h0 = th * TH, ps0 = td * TD;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int m = item_meta[r];
      const int pair = m & 0xff, hy = (m >> 8) & 0xff, dz = (m >> 16) & 0xff;
      const int p_in = ps0 - a.out.hlo + dz - 1;
      const int64_t gq = a.in.doff + p_in;
      const int sp = p_in + a.in.hlo;
      const int h = h0 + hy - 1, w = w0 - 2 + 2 * pair;
      const bool ok = (m >> 24) && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H && w >= 0 && w + 1 < W;
      voff[r] = ok ? 2 * (sp * (int)a.in.plane + h * W + w) : BUF_OOB;
    }
    n_plan = n;
  };

  uint32_t v[ROUNDS][8];
  // part `q` of 3 of one group of 8 input channels of chunk c for the planned tile (`live` false: nothing to fetch, all
  // loads out of range).  A group is requested over three steps so that no request queue ever holds a long batch in
  // front of the weight fragments (vector loads return in order).
  auto load_part = [&](int c, int cig, int q, bool live) {
    const __amdgpu_buffer_rsrc_t rs_in = make_rsrc(in + n_plan * a.in.nstride, (uint32_t)a.in.nstride * 2);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (e / 3 != q) continue;                      // channels 0-2, 3-5, 6-7
      const int ch = c * CI_CHUNK + cig * 8 + e;
      const bool chan_ok = live && ch < a.cin_k;     // wave-uniform
      const int soff = __builtin_amdgcn_readfirstlane(chan_ok ? 2 * ch * (int)a.in.cstride : 0);
#pragma unroll
      for (int r = 0; r < ROUNDS; ++r) v[r][e] = __builtin_amdgcn_raw_buffer_load_b32(rs_in, chan_ok ? voff[r] : BUF_OOB, soff, 0);
    }
  };
  auto load_half = [&](int c, int cig, bool live) {
    load_part(c, cig, 0, live);
    load_part(c, cig, 1, live);
    load_part(c, cig, 2, live);
  };
  auto store_half = [&](int buf, int cig) {
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      if (!(item_meta[r] >> 24)) continue;
      uint4 u0, u1;
      u0.x = __builtin_amdgcn_perm(v[r][1], v[r][0], 0x05040100); u1.x = __builtin_amdgcn_perm(v[r][1], v[r][0], 0x07060302);
      u0.y = __builtin_amdgcn_perm(v[r][3], v[r][2], 0x05040100); u1.y = __builtin_amdgcn_perm(v[r][3], v[r][2], 0x07060302);
      u0.z = __builtin_amdgcn_perm(v[r][5], v[r][4], 0x05040100); u1.z = __builtin_amdgcn_perm(v[r][5], v[r][4], 0x07060302);
      u0.w = __builtin_amdgcn_perm(v[r][7], v[r][6], 0x05040100); u1.w = __builtin_amdgcn_perm(v[r][7], v[r][6], 0x07060302);
      uint4* dst = lds + buf * BUF_UNITS + cig * CIG_UNITS + lds_unit[r];
      dst[0] = u0;
      dst[1] = u1;
    }
  };

  const int j = lane & 31;
  // The accumulators of a tile start from the bias (the sums are then taken in the order of the kernel above: same
  // bits).  Writing 256 accumulation registers one by one from the vector ALU costs a wavefront about 5000 cycles
  // per tile (measured); instead the bias enters as a product: a weight-shaped fragment that holds, for each channel
  // of the block, the three bfloat16 pieces of its fp32 bias (upper, middle and lower 8 mantissa bits, cut by
  // truncation: their sum is the bias exactly) in the first three of the 16 contraction slots and zeros in the others,
  // multiplied by a fragment of ones: sixteen extra MFMAs per tile, D = hi + mid + lo + 0 ... = bias in every column.
  uint4* biasf_l = lds + 2 * BUF_UNITS + wcb * CB * 64;       // [WCB][CB][64 lanes] fragments behind the two stage buffers
  if ((tid & 255) < CB * 64) {
    const int cb = (tid & 255) >> 6, l = tid & 63;
    uint4 f = {0u, 0u, 0u, 0u};
    const int co = (co_blk0 + cb) * 32 + l;
    if (l < 32 && bias && co < a.cout_k) {
      const float bv = bias[co];
      const uint32_t hi = __float_as_uint(bv) & 0xffff0000u;
      const float r1 = bv - __uint_as_float(hi);
      const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
      const float r2 = r1 - __uint_as_float(mid);
      const uint32_t lo = __float_as_uint(r2) & 0xffff0000u;
      f.x = (hi >> 16) | mid;
      f.y = lo >> 16;
    }
    biasf_l[tid & 255] = f;
  }
  __syncthreads();
  f32x16 acc[CB][VB];
  auto init_acc = [&]() {
    const uint4 ones_u = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_u);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const bf16x8 bf = __builtin_bit_cast(bf16x8, biasf_l[cb * 64 + lane]);
#pragma unroll
      for (int b = 0; b < VB; ++b) acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, ones, zero, 0, 0, 0);
    }
  };
  init_acc();

  const int lane_unit = (lane >> 5) * CIG_UNITS + (wd * TH2 + rh * VB) * P + j + 1;
  const int a_voff = lane * 16;
  // weight fragments of one (kd,kw) step: [kh][channel block]; a channel block beyond Cout re-reads the last valid one
  auto load_a = [&](int c, int step, uint4 (&dst)[3][CB]) {
    const int kd = step / 3, kw = step % 3;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const int blk = min(co_blk0 + cb, a.ncoblk - 1);
#pragma unroll
      for (int kh = 0; kh < 3; ++kh) {
        const int soff = __builtin_amdgcn_readfirstlane(((blk * a.nchunks + c) * 27 + kd * 9 + kh * 3 + kw) * 1024);
        const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rs_w, a_voff, soff, 0);
        dst[kh][cb] = uint4{t.x, t.y, t.z, t.w};
      }
    }
  };

  uint4 afr[2][3][CB];        // weight fragments of the current and of the next step
  const int G = gridDim.x;
  int tile = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  if (tile >= a.ntiles) return;
  const int nch = a.nchunks;

  // One chunk: 9 steps of 24 * CB products.  c_next: the chunk whose weight stream follows this one's.  The step order
  // is: request the next step's weight fragments, then this step's share of the next stage's input, then multiply; a
  // row fragment register is refilled for the next step as soon as its last product has been issued.
  auto compute_chunk = [&](int c, int c_next, int buf, bool more, int next_tile, bool last_chunk) {
    const uint4* base = lds + buf * BUF_UNITS + lane_unit;
    uint4 bfr[NFRAG];
#pragma unroll
    for (int s = 0; s < NFRAG; ++s) bfr[s] = base[s * P];
    const int cn = last_chunk ? 0 : c + 1;
#pragma unroll
    for (int step = 0; step < 9; ++step) {
      if (step + 1 < 9) load_a(c, step + 1, afr[(step + 1) & 1]);
      else load_a(c_next, 0, afr[(step + 1) & 1]);
      if (step == 0 && last_chunk && more) plan_tile(next_tile);
      if (step < 3) load_part(cn, 0, step, more);
      if (step == 4 && more) store_half(buf ^ 1, 0);
      if (step >= 4 && step < 7) load_part(cn, 1, step - 4, more);
      const int kd1 = (step + 1) / 3, kw1 = (step + 1) % 3;
#pragma unroll
      for (int s = 0; s < NFRAG; ++s) {
        const bf16x8 B = __builtin_bit_cast(bf16x8, bfr[s]);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
          const int b = s - kh;
          if (b >= 0 && b < VB) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
              acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afr[step & 1][kh][cb]), B, acc[cb][b], 0, 0, 0);
          }
        }
        if (step + 1 < 9) bfr[s] = base[(kd1 * TH2 + s) * P + kw1];
      }
      // one wavefront per SIMD: the requests, address arithmetic and LDS traffic of the step must be issued in the
      // shadow of its products (a product occupies the matrix pipe for 32 cycles, the wavefront can issue about seven
      // other instructions meanwhile), not in a block in front of them
#pragma unroll
      for (int i = 0; i < 3 * VB * CB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x326, 3, 0);      // up to three of: VALU, SALU, vector-memory read, LDS read / write
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) store_half(buf ^ 1, 1);
    // nine steps: the fragments requested at step 8 sit in set 1, the next chunk starts with set 0
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) afr[0][kh][cb] = afr[1][kh][cb];
  };

  // Epilogue of a tile (CB * 128 values per lane): everything that does not depend on the value is taken out of the
  // per-value path.  Activation as med3(v, slope * v, +inf) (the same bits as "v > 0 ? v : slope * v" for
  // 0 <= slope <= 1), skipped when there is none.
  auto epilogue = [&](int tile_) {
    int t = tile_;
    const int tw = t % a.tiles_w; t /= a.tiles_w;
    const int th = t % a.tiles_h; t /= a.tiles_h;
    const int td = t % a.tiles_d;
    const int n = t / a.tiles_d;
    const int w0 = tw * TW, h0 = th * TH + rh * VB, ps = td * TD + wd;      // this wavefront's first row
    if (ps >= a.out.ds) return;
    const int64_t gp = a.out.doff + ps - a.out.hlo;
    const bool inside = gp >= 0 && gp < a.out.dglob;
    const int row_ch = 4 * (lane >> 5);
    const __amdgpu_buffer_rsrc_t rs_out = make_rsrc(out + n * a.out.nstride, (uint32_t)a.out.nstride * 2);
    // A lane holds one voxel of 16 channels; a store wants two neighbouring voxels of one channel.  Each lane packs
    // its channel pair (r, r+1) to bf16, fetches its neighbour's packed pair (lanes 2k and 2k+1 hold voxels 2k and
    // 2k+1) and picks, with a per-lane byte selector, channel r of both voxels (even lane) or channel r+1 of both
    // (odd lane): one conversion, one lane exchange and one byte permute per stored dword, no selects.
    const bool odd = lane & 1;
    const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
    const int cs2 = 2 * (int)a.out.cstride;
    const int vbase = (row_ch + (odd ? 1 : 0)) * cs2 + 2 * (ps * (int)a.out.plane + h0 * W + w0 + j - (odd ? 1 : 0));
    const bool w_ok = w0 + j - (odd ? 1 : 0) < W;
    const bool act = a.out_slope != 1.f;        // wave-uniform
    const float slope = a.out_slope;
    const float inf = __builtin_inff();
    // ACT / WHOLE are wave-uniform facts: one branch per channel block, not one select per value
    auto block = [&](int cb, auto act_c, auto whole_c) {
      constexpr bool ACT = decltype(act_c)::value, WHOLE = decltype(whole_c)::value;
      const int cblk = co_blk0 + cb;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const int co_u = cblk * 32 + 8 * (r / 4) + (r % 4);
        const int soff = __builtin_amdgcn_readfirstlane(co_u * cs2);
        const bool ch_ok = WHOLE || co_u + row_ch + (odd ? 1 : 0) < a.cout_k;
#pragma unroll
        for (int b = 0; b < VB; ++b) {
          float v0 = acc[cb][b][r], v1 = acc[cb][b][r + 1];
          if (ACT) {      // max(v, slope v): v where v > 0, slope v elsewhere (0 <= slope <= 1)
            const float s0 = v0 * slope, s1 = v1 * slope;
            asm("v_max_f32 %0, %1, %2" : "=v"(v0) : "v"(v0), "v"(s0));
            asm("v_max_f32 %0, %1, %2" : "=v"(v1) : "v"(v1), "v"(s1));
          }
          const uint32_t own = pack_bf16x2(v0, v1);
          const uint32_t nb = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0xB1, 0xF, 0xF, true);
          uint32_t pk = __builtin_amdgcn_perm(nb, own, sel);
          int o = (w_ok && h0 + b < H) ? vbase + 2 * b * W : BUF_OOB;
          if (!WHOLE) {
            pk = inside ? pk : 0u;
            o = ch_ok ? o : BUF_OOB;
          }
          __builtin_amdgcn_raw_buffer_store_b32(pk, rs_out, o, soff, 0);
        }
      }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const int cblk = co_blk0 + cb;
      if (cblk >= a.ncoblk) continue;
      const bool whole = cblk * 32 + 32 <= a.cout_k && inside;     // the common case
      if (whole) {
        if (act) block(cb, T_{}, T_{});
        else block(cb, F_{}, T_{});
      } else {
        block(cb, T_{}, F_{});       // (slope 1 leaves the values as they are)
      }
    }
  };

  // prologue: first stage into buffer 0, first two steps of the weight stream
  plan_tile(tile);
  load_half(0, 0, true);
  store_half(0, 0);
  load_half(0, 1, true);
  store_half(0, 1);
  load_a(0, 0, afr[0]);
  __syncthreads();
  int buf = 0;
  while (true) {
    const int next_tile = tile + G;
    for (int c = 0; c < nch; ++c) {
      const bool last_chunk = c + 1 == nch;
      const bool more = !last_chunk || next_tile < a.ntiles;
      compute_chunk(c, last_chunk ? 0 : c + 1, buf, more, next_tile, last_chunk);
      __syncthreads();
      buf ^= 1;
    }
    epilogue(tile);
    init_acc();
    tile = next_tile;
    if (tile >= a.ntiles) break;
  }
}

// out = act(bias + sum over splits of part[split]) in split order; planes outside the global volume are zero.
// part holds raw accumulator tiles (see the SPLIT epilogue): an output element (n, co, ps, h, w) is register
// b*16 + r of lane `lane` of the wavefront (channel block co/32, plane ps % ND) of tile (n, ps/ND, h/TH, w/TW).
struct SplitGeo {
  int nd, twc, rpb, ncoblk, tiles_w, tiles_h, tiles_d, ntiles;
};
__global__ void __launch_bounds__(256) conv_split_reduce_kernel(const float* __restrict__ part, const float* __restrict__ bias,
                                                                bf16_t* __restrict__ out, Geo g, SplitGeo q, int splits, float slope) {
  const int64_t total = (int64_t)g.n * g.nstride;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int64_t t = i;
  const int w = (int)(t % g.w); t /= g.w;
  const int h = (int)(t % g.h); t /= g.h;
  const int ps = (int)(t % g.ds); t /= g.ds;
  const int co = (int)(t % g.c);
  const int n = (int)(t / g.c);
  const int th_rows = 4 * q.rpb;
  const int tile = ((n * q.tiles_d + ps / q.nd) * q.tiles_h + h / th_rows) * q.tiles_w + w / q.twc;
  const int hl = h % th_rows, wl = w % q.twc, c32 = co % 32;
  const int b = hl / q.rpb, j = (hl % q.rpb) * q.twc + wl;
  const int r = 4 * (c32 / 8) + c32 % 4, lane = ((c32 / 4) % 2) * 32 + j;
  const int64_t slot = ((((int64_t)tile * q.ncoblk + co / 32) * q.nd + ps % q.nd) * 64 + (b * 16 + r)) * 64 + lane;
  const int64_t per_split = (int64_t)q.ntiles * q.ncoblk * q.nd * 4096;
  float s = 0.f;
  for (int sp = 0; sp < splits; ++sp) s += part[sp * per_split + slot];
  const int64_t gp = g.doff + ps - g.hlo;
  float v = s + (bias ? bias[co] : 0.f);
  if (!(v > 0.f)) v *= slope;
  out[i] = f32_to_bf16((gp >= 0 && gp < g.dglob) ? v : 0.f);
}

// How many ways the input-channel chunks are split: 1 unless the tiles alone would leave most CUs idle.
static int mfma_splits(const h3d_tensor* in, const h3d_tensor* out) {
  const int nchunks = (int)cdiv(in->c, CI_CHUNK), ncoblk = (int)cdiv(out->c, 32);
  const bool wide = out->w > 16, two_cb = out->c > 32;
  const int twc = wide ? 32 : 16, ncb = two_cb ? 2 : 1, nd = 8 / ncb, th = 4 * (32 / twc);
  const int64_t ds = out->halo_lo + out->d + out->halo_hi;
  const int64_t wgs = (int64_t)out->n * cdiv(ds, nd) * cdiv(out->h, th) * cdiv(out->w, twc) * cdiv(ncoblk, ncb);
  if (wide || wgs == 0 || wgs >= 64 || nchunks < 2 || !is_packed(out)) return 1;    // (only the narrow-volume variants come in a split form)
  int s = (int)std::min<int64_t>(nchunks, cdiv(256, wgs));
  const int64_t out_elems = (int64_t)out->n * out->c * ds * out->h * out->w;
  (void)out_elems;
  {
    const int64_t padded = (int64_t)out->n * cdiv(ds, nd) * cdiv(out->h, 8) * cdiv(out->w, 16) * ncoblk * nd * 4096;
    while (s > 1 && s * padded * 4 > ((int64_t)24 << 20)) --s;   // the partials cost a write and a read
  }
  const int cps = (int)cdiv(nchunks, s);
  return (int)cdiv(nchunks, cps);
}

bool mfma_fwd_supported(const h3d_tensor* in, const h3d_tensor* out) {
  if (in->dtype != H3D_BF16) return false;
  if (in->c < 1 || out->c < 1) return false;
  // 32-bit in-sample offsets inside the kernel
  // buffer loads address a whole sample (all channels) with 31-bit byte offsets
  return sample_span(in) < ((int64_t)1 << 30) && sample_span(out) < ((int64_t)1 << 30);
}

static void wp_dims(int cin_k, int cout_k, int* nchunks, int* ncoblk) {
  *nchunks = (int)cdiv(cin_k, CI_CHUNK);
  *ncoblk = (int)cdiv(cout_k, 32);
}

// floats of ONE split's partial tiles: the split kernels are the narrow-volume instances (16-column blocks, 8 rows)
static size_t split_part_floats(const h3d_tensor* out) {
  const int ncoblk = (int)cdiv(out->c, 32), nd = out->c > 32 ? 4 : 8;
  const int64_t ds = out->halo_lo + out->d + out->halo_hi;
  return (size_t)((int64_t)out->n * cdiv(ds, nd) * cdiv(out->h, 8) * cdiv(out->w, 16)) * ncoblk * nd * 4096;
}

static size_t mfma_wp_bytes(const h3d_tensor* in, const h3d_tensor* out) {
  int nchunks, ncoblk;
  wp_dims(in->c, out->c, &nchunks, &ncoblk);
  return ((size_t)ncoblk * nchunks * 27 * 512 * sizeof(bf16_t) + 255) & ~(size_t)255;
}

bool conv3d_thin_supported(const h3d_tensor* in, const h3d_tensor* out);
h3d_status conv3d_thin(void* handle, const h3d_tensor* in, const void* w, const float* bias, h3d_tensor* out, bool transpose,
                       float out_slope, void* ws, hipStream_t stream);

// Backward-data onto at most 4 channels from 17 to 32 (the first layer of the U-Net-shaped level: 32 -> 1): the
// row-streaming thin kernel holds 16 input channels in its LDS ring, so the sum over the channels is taken in two
// passes, channels 0-15 into dx and the rest into a buffer of dx's size in the workspace, and the two are added:
// dx = bf16(bf16(sum over the first 16) + bf16(sum over the others)), one rounding more than a single pass.
// `in` is split into two channel-range views; both must be shapes of the row-streaming variant.
constexpr size_t THIN2_WP_BYTES = 16384;
static bool thin_two_pass_shape(const h3d_tensor* in, const h3d_tensor* out, h3d_tensor* ia, h3d_tensor* ib) {
  if (in->dtype != H3D_BF16 || in->c <= 16 || in->c > 32 || out->c < 1 || out->c > 4 || !is_packed(out)) return false;
  if (in->w % 8 || out->h < 8 || (uintptr_t)in->data % 16 || (out->data && (uintptr_t)out->data % 16)) return false;
  const Geo g = make_geo(in);
  if (g.cstride % 8) return false;
  h3d_tensor a = *in, b = *in;
  a.c = 16; a.c_stride = g.cstride; a.n_stride = g.nstride;
  b.c = in->c - 16; b.c_stride = g.cstride; b.n_stride = g.nstride;
  b.data = in->data ? (void*)((bf16_t*)in->data + 16 * g.cstride) : nullptr;
  if (!conv3d_thin_supported(&a, out) || !conv3d_thin_supported(&b, out)) return false;
  if (ia) *ia = a;
  if (ib) *ib = b;
  return true;
}
static size_t thin_two_pass_ws_bytes(const h3d_tensor* out) {
  return THIN2_WP_BYTES + (size_t)out->n * out->c * (out->halo_lo + out->d + out->halo_hi) * out->h * out->w * sizeof(bf16_t);
}
// dst[i] = bf16(dst[i] + src[i]), 8 elements per thread (n8 groups), then the tail one by one
__global__ void __launch_bounds__(256) add_bf16_kernel(bf16_t* __restrict__ dst, const bf16_t* __restrict__ src, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i + 8 <= n) {
    uint4 a = *reinterpret_cast<const uint4*>(dst + i);
    const uint4 b = *reinterpret_cast<const uint4*>(src + i);
    auto add2 = [](uint32_t x, uint32_t y) {
      return pack_bf16x2(__uint_as_float(x << 16) + __uint_as_float(y << 16),
                         __uint_as_float(x & 0xffff0000u) + __uint_as_float(y & 0xffff0000u));
    };
    a.x = add2(a.x, b.x); a.y = add2(a.y, b.y); a.z = add2(a.z, b.z); a.w = add2(a.w, b.w);
    *reinterpret_cast<uint4*>(dst + i) = a;
  } else {
    for (int64_t j = i; j < n; ++j) dst[j] = f32_to_bf16(bf16_to_f32(dst[j]) + bf16_to_f32(src[j]));
  }
}

size_t mfma_fwd_ws_bytes(const h3d_tensor* in, const h3d_tensor* out) {
  size_t b = mfma_wp_bytes(in, out);
  if (thin_two_pass_shape(in, out, nullptr, nullptr)) b = std::max(b, thin_two_pass_ws_bytes(out));
  const int s = mfma_splits(in, out);
  if (s > 1) b += (size_t)s * split_part_floats(out) * sizeof(float);
  return b;
}

template <int NCB, int ND, int TWC, bool MASKED, bool VEC, bool SPLIT = false, bool FLAT = false>
static h3d_status launch_variant(void* handle, const bf16_t* in, const bf16_t* mask, const uint4* wp, const float* bias,
                                 bf16_t* out, MfmaArgs a, int n, hipStream_t stream) {
  constexpr int RPB = 32 / TWC, TH = 4 * RPB;
  constexpr int P = TWC == 32 ? 36 : 20;
  constexpr int TDP = FLAT ? 1 : ND, THT = FLAT ? TH * ND : TH;
  constexpr size_t lds_bytes = (size_t)2 * 2 * (TDP + 2) * (THT + 2) * P * 16;
  a.tiles_w = (int)cdiv(a.out.w, TWC);
  a.tiles_h = (int)cdiv(a.out.h, THT);
  a.tiles_d = (int)cdiv(a.out.ds, TDP);
  int64_t ntiles = (int64_t)n * a.tiles_d * a.tiles_h * a.tiles_w;
  int64_t gy = cdiv(a.ncoblk, NCB);
  if (ntiles >= ((int64_t)1 << 31) || gy > 65535) return fail(handle, H3D_EINVAL, "conv3d: too many workgroups");
  a.ntiles = (int)ntiles;
  // one resident workgroup per CU (LDS-limited), spread over the output-channel groups
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  int64_t gx = std::min<int64_t>(ntiles, std::max<int64_t>(1, num_cu / (gy * a.csplit)));
  auto kern = conv3d_mfma_kernel<NCB, ND, TWC, MASKED, VEC, SPLIT, FLAT>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d: cannot raise the dynamic LDS limit to %zu bytes", lds_bytes);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)gx, (unsigned)gy, (unsigned)a.csplit), dim3(WG_THREADS), lds_bytes, stream, in, mask, wp,
                     a.csplit > 1 ? nullptr : bias, out, a);
  note_kernel(handle, "conv3d_mfma_kernel<%d,%d,%d,%d,%d,%d,%d>", NCB, ND, TWC, (int)MASKED, (int)VEC, (int)SPLIT, (int)FLAT);
  if (a.csplit > 1) return hipGetLastError() == hipSuccess ? H3D_OK : fail(handle, H3D_EHIP, "conv3d_mfma: launch failed");
  return launch_status(handle, "conv3d_mfma");
}

static bool wide_shape(const MfmaArgs& a) {
  return a.out.w > 16 && a.out.ds >= 3 && a.out.h >= 4 && a.csplit == 1;
}

template <int CB, int WCB = 1, int RSP = 1>
static h3d_status launch_wide(void* handle, const bf16_t* in, const uint4* wp, const float* bias, bf16_t* out, MfmaArgs a, int n,
                              hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)2 * 2 * 6 * 10 * 36 * 16 + WCB * CB * 64 * 16;     // two stage buffers + the bias fragments
  a.tiles_w = (int)cdiv(a.out.w, 32);
  a.tiles_h = (int)cdiv(a.out.h, 8);
  a.tiles_d = (int)cdiv(a.out.ds, 4);
  const int64_t ntiles = (int64_t)n * a.tiles_d * a.tiles_h * a.tiles_w;
  const int64_t gy = cdiv(a.ncoblk, CB * WCB);
  if (ntiles >= ((int64_t)1 << 31) || gy > 65535) return fail(handle, H3D_EINVAL, "conv3d: too many workgroups");
  a.ntiles = (int)ntiles;
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  const int64_t gx = std::min<int64_t>(ntiles, std::max<int64_t>(1, num_cu / gy));
  auto kern = conv3d_mfma_wide_kernel<CB, WCB, RSP>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d: cannot raise the dynamic LDS limit to %zu bytes", lds_bytes);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)gx, (unsigned)gy), dim3(256 * WCB * RSP), lds_bytes, stream, in, wp, bias, out, a);
  if (WCB * RSP == 1) note_kernel(handle, "conv3d_mfma_wide_kernel<%d>", CB);
  else if (RSP == 1) note_kernel(handle, "conv3d_mfma_wide_kernel<%d,%d>", CB, WCB);
  else note_kernel(handle, "conv3d_mfma_wide_kernel<%d,%d,%d>", CB, WCB, RSP);
  return launch_status(handle, "conv3d_mfma_wide");
}

template <bool MASKED, bool VEC>
static h3d_status pick_variant(void* handle, const bf16_t* in, const bf16_t* mask, const uint4* wp, const float* bias,
                               bf16_t* out, const MfmaArgs& a, int n, hipStream_t s) {
  const bool wide = a.out.w > 16;
  const bool two_cb = a.cout_k > 32;
  // one- or two-plane outputs with more than 32 channels and enough rows: the row-group layout
  const bool flat = two_cb && a.out.ds <= 2 && a.csplit == 1;
  if (flat && wide && a.out.h >= 16) return launch_variant<2, 4, 32, MASKED, VEC, false, true>(handle, in, mask, wp, bias, out, a, n, s);
  if (flat && !wide && a.out.h >= 32) return launch_variant<2, 4, 16, MASKED, VEC, false, true>(handle, in, mask, wp, bias, out, a, n, s);
  if (wide) {
    return two_cb ? launch_variant<2, 4, 32, MASKED, VEC>(handle, in, mask, wp, bias, out, a, n, s)
                  : launch_variant<1, 8, 32, MASKED, VEC>(handle, in, mask, wp, bias, out, a, n, s);
  }
  if (a.csplit > 1)
    return two_cb ? launch_variant<2, 4, 16, MASKED, VEC, true>(handle, in, mask, wp, bias, out, a, n, s)
                  : launch_variant<1, 8, 16, MASKED, VEC, true>(handle, in, mask, wp, bias, out, a, n, s);
  return two_cb ? launch_variant<2, 4, 16, MASKED, VEC>(handle, in, mask, wp, bias, out, a, n, s)
                : launch_variant<1, 8, 16, MASKED, VEC>(handle, in, mask, wp, bias, out, a, n, s);
}

h3d_status conv3d_mfma(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                       h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                       hipStream_t stream) {
  MfmaArgs a;
  a.in = make_geo(in);
  a.mask = mask ? make_geo(mask) : a.in;
  a.out = make_geo(out);
  a.cin_k = in->c; a.cout_k = out->c;
  wp_dims(a.cin_k, a.cout_k, &a.nchunks, &a.ncoblk);
  a.out_slope = out_slope; a.mask_slope = mask_slope;
  if ((int64_t)out->n * a.out.ds * out->h * out->w == 0) return H3D_OK;
  if (!ws || ws_bytes < mfma_fwd_ws_bytes(in, out)) return fail(handle, H3D_EWORKSPACE, "conv3d: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d: workspace must be 16-byte aligned");
  // a handful of output channels from at most 16 input channels: the tap-row-folding kernel
  if (!mask && conv3d_thin_supported(in, out)) return conv3d_thin(handle, in, w, bias, out, transpose, out_slope, ws, stream);
  // .. from 17 to 32 channels, backward-data without bias and activation: two passes of it
  h3d_tensor ia, ib;
  if (!mask && transpose && !bias && out_slope == 1.f && thin_two_pass_shape(in, out, &ia, &ib)) {
    h3d_tensor tmp = *out;
    tmp.data = static_cast<char*>(ws) + THIN2_WP_BYTES;
    H3D_TRY(conv3d_thin(handle, &ia, w, nullptr, out, true, 1.f, ws, stream));
    // transposed packing reads w[c][m][tap] with c the channel of `in`: the second half starts 16 rows further on
    H3D_TRY(conv3d_thin(handle, &ib, (const bf16_t*)w + (size_t)16 * out->c * 27, nullptr, &tmp, true, 1.f, ws, stream));
    const int64_t n = (int64_t)out->n * a.out.nstride;
    hipLaunchKernelGGL(add_bf16_kernel, dim3((unsigned)cdiv(cdiv(n, 8), 256)), dim3(256), 0, stream, (bf16_t*)out->data,
                       (const bf16_t*)tmp.data, n);
    note_kernel(handle, "conv3d_thin_roll (two passes)");
    return launch_status(handle, "conv3d_thin_two_pass");
  }
  const bool vec = (in->w % 2 == 0) && ((uintptr_t)in->data % 4 == 0) && ((uintptr_t)out->data % 4 == 0) &&
                   (!mask || (uintptr_t)mask->data % 4 == 0);
  const int cin = transpose ? a.cout_k : a.cin_k, cout = transpose ? a.cin_k : a.cout_k;
  int64_t total = (int64_t)a.ncoblk * a.nchunks * 27 * 512;
  hipLaunchKernelGGL(pack_w_mfma_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws, cin,
                     cout, transpose ? 1 : 0, a.nchunks, a.ncoblk);
  const bf16_t* ip = (const bf16_t*)in->data;
  const bf16_t* mp = mask ? (const bf16_t*)mask->data : nullptr;
  bf16_t* op = (bf16_t*)out->data;
  const uint4* wq = (const uint4*)ws;
  a.csplit = mfma_splits(in, out);
  a.chunks_per_split = (int)cdiv(a.nchunks, a.csplit);
  a.part = a.csplit > 1 ? reinterpret_cast<float*>(static_cast<char*>(ws) + mfma_wp_bytes(in, out)) : nullptr;
  h3d_status st;
  if (!mask && vec && wide_shape(a)) {
    if (a.cout_k > 32) {
      // few tiles (a small volume): one channel block per workgroup doubles the workgroups, same sums in the same order
      const int64_t ntiles = (int64_t)out->n * cdiv(a.out.ds, 4) * cdiv(a.out.h, 8) * cdiv(a.out.w, 32);
      const int num_cu = static_cast<Handle*>(handle)->num_cu;
      if (ntiles * cdiv(a.ncoblk, 2) * 4 < (int64_t)num_cu * 3) return launch_wide<1, 1>(handle, ip, wq, bias, op, a, out->n, stream);
      return launch_wide<1, 2>(handle, ip, wq, bias, op, a, out->n, stream);
    }
    if (a.cin_k > 8) {      // (16 input channels = one chunk per tile: 16->32 on 4 x 64^3 0.056 ms with the kernel above, 0.043 here)
      // one block of output channels: with short channel loops (at most 32 input channels) or few tiles the eight-wavefront
      // form that splits the rows of a plane measured faster (32->16 on 4 x 64^3 0.068 -> 0.062 ms, 32->1 on the U-Net
      // shard 0.239 -> 0.222), with four chunks and many tiles slower (64->32 on the U-Net shard 0.480 -> 0.490)
      const int64_t ntiles = (int64_t)out->n * cdiv(a.out.ds, 4) * cdiv(a.out.h, 8) * cdiv(a.out.w, 32);
      if (a.nchunks <= 2 || ntiles < 2 * static_cast<Handle*>(handle)->num_cu)
        return launch_wide<1, 1, 2>(handle, ip, wq, bias, op, a, out->n, stream);
      return launch_wide<1, 1>(handle, ip, wq, bias, op, a, out->n, stream);
    }
  }
  if (mask) st = vec ? pick_variant<true, true>(handle, ip, mp, wq, bias, op, a, out->n, stream)
                     : pick_variant<true, false>(handle, ip, mp, wq, bias, op, a, out->n, stream);
  else st = vec ? pick_variant<false, true>(handle, ip, mp, wq, bias, op, a, out->n, stream)
                : pick_variant<false, false>(handle, ip, mp, wq, bias, op, a, out->n, stream);
  if (st != H3D_OK || a.csplit == 1) return st;
  const int64_t out_total = (int64_t)out->n * a.out.nstride;
  SplitGeo q;
  q.nd = a.cout_k > 32 ? 4 : 8; q.twc = 16; q.rpb = 2; q.ncoblk = a.ncoblk;
  q.tiles_w = (int)cdiv(a.out.w, 16); q.tiles_h = (int)cdiv(a.out.h, 8); q.tiles_d = (int)cdiv(a.out.ds, q.nd);
  q.ntiles = out->n * q.tiles_d * q.tiles_h * q.tiles_w;
  hipLaunchKernelGGL(conv_split_reduce_kernel, dim3((unsigned)cdiv(out_total, 256)), dim3(256), 0, stream, (const float*)a.part, bias, op,
                     a.out, q, a.csplit, out_slope);
  return launch_status(handle, "conv3d_split_reduce");
}

}  // namespace h3d
