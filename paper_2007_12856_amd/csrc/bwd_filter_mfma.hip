// Backward-filter (BF pass, Sec. III-C) on the matrix cores, bf16 in / fp32 accumulate.
//
//   dW[co][ci,kd,kh,kw] = sum over voxels v of g[co][v] * x~[ci][v + (kd,kh,kw) - 1]
//
// is a GEMM whose contraction runs over VOXELS: with v_mfma_f32_16x16x32_bf16 a lane feeds 8
// consecutive voxels along W of one row (A: a channel of g) or one column (B: a shifted channel of
// x) — contiguous 16 bytes in NCDHW, so both operands keep their natural layout (no transpose).
//   * rows    = output channels, in blocks of 16;
//   * columns = (ci, kd, kh) combinations, ci slowest, in blocks of 16; the three kw taps of a
//     combination are three MFMAs fed from ONE aligned 16-byte LDS read: the kw = 0 / 2 operands are
//     that block shifted by one element, completed with the neighbouring lane group's edge dword
//     (ds_bpermute) or, at the ends of a row segment, one dword read from the tile's halo;
//   * LDS pitches of the x tile are chosen so that the 16 combinations of a column block fall into
//     16 distinct 16-byte bank groups (row pitch r odd, plane pitch = 3r, channel pitch = 9r mod 16);
//   * a workgroup = 3 wavefronts x 3 column blocks = the 144 combinations of 16 input channels,
//     times RBW row blocks; it streams a fixed chunk of voxel tiles through LDS and keeps the whole
//     dW tile in accumulators;
//   * db[co] = sum g comes from one extra MFMA per A fragment against an all-ones operand.
// Determinism: the split of the voxel range into chunks and tiles is fixed by the shape; every
// workgroup writes its partial tile; a second kernel adds the chunk partials in chunk order.
#include <algorithm>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BF_OOB = (int)0x80000000;   // byte offset beyond every buffer: such a lane transfers zeros

__device__ __forceinline__ h3d_i32x4 bf_rsrc(const void* base, uint32_t bytes) { return lds_dma_rsrc(base, bytes); }
// the same range as a resource of the compiler's own buffer loads (global -> registers)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t bf_rsrc_reg(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                           (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

// 64 lanes x 16 bytes from per-lane buffer offsets straight into 1 KB of LDS at `lds_dst` (wave-uniform); issued so that
// the compiler does not wait for it before later LDS reads (common.h): every kernel here waits and synchronises itself
__device__ __forceinline__ void dma16(h3d_i32x4 rs, uint4* lds_dst, int voff) { lds_dma16(rs, lds_addr_of(lds_dst), voff); }
// the same copy through the compiler's builtin: the compiler then waits for it before the next LDS read.  Kept for the
// one-row-group, 16-channel instances of the rolling kernel, which measured faster this way (16 -> 32 channels on
// 4 x 64^3: 0.066 against 0.077 ms)
__device__ __forceinline__ void dma16_visible(h3d_i32x4 rs, uint4* lds_dst, int voff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(
      __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)(uint32_t)rs[1] << 32) | (uint32_t)rs[0]), 0, rs[2], 0x00020000),
      (__attribute__((address_space(3))) void*)lds_dst, 16, voff, 0, 0, 0);
}

constexpr int cmod_ge(int lo, int target_mod16) {  // smallest v >= lo with v % 16 == target_mod16
  int v = lo;
  while (v % 16 != target_mod16) ++v;
  return v;
}

template <int TW, int TH>
struct BfTile {
  static constexpr int GW = TW >= 32 ? 4 : TW / 8;        // lane groups (of 8 voxels) side by side in a row
  static constexpr int RPK = TW >= 32 ? 1 : 32 / TW;      // rows per K-step of 32 voxels
  static constexpr int KS_PER_ROW = TW >= 32 ? TW / 32 : 1;
  static constexpr int KSTEPS = TH * TW / 32;
  static constexpr int XU = TW / 8 + 2;                   // x row: w in [w0-8, w0+TW+8)
  static constexpr int PR = XU | 1;
  static constexpr int PD = cmod_ge((TH + 2) * PR, (3 * PR) % 16);
  static constexpr int PC = cmod_ge(3 * PD, (9 * PR) % 16);
  static constexpr int GU = TW / 8;
  static constexpr int PG = (TH * GU) | 1;
  static constexpr int X_UNITS = 16 * PC;
};

struct BfmArgs {
  Geo x, g, z;
  int cin, cout;
  int tiles_w, tiles_h;       // tiles per plane
  int64_t ntiles;             // n * d * tiles_h * tiles_w
  int tiles_per_chunk, nchunks;
  int gy, gz;                 // output-channel groups and input-channel groups of the grid
  int wpair;                  // rolling kernel: 2 = the two 32-column tiles that share 128-byte lines go to two
                              // neighbouring workgroups (same XCD, same time), which write separate partials
  int npart;                  // partial tiles in the workspace = nchunks * wpair
  float mask_slope;
  int vec_ok;                 // W % 8 == 0 and 16-byte aligned bases: whole units are loaded at once
  int dma_ok;                 // every sample fits 31-bit byte offsets: tiles can be moved by buffer loads into LDS
};

__device__ __forceinline__ uint4 load_unit(const bf16_t* base, int w, int W, bool row_ok, bool vec, int w0) {
  // 8 elements at absolute columns w..w+7 of a row; `base` points at column w0 of that row.
  // Zero where outside [0,W) or the row is invalid.
  uint4 u = {0, 0, 0, 0};
  if (!row_ok) return u;
  base += w - w0;
  if (vec) {
    if (w >= 0 && w + 8 <= W) u = *reinterpret_cast<const uint4*>(base);
    return u;
  }
  uint32_t e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = (w + i >= 0 && w + i < W) ? base[i] : 0;
  u.x = e[0] | (e[1] << 16); u.y = e[2] | (e[3] << 16); u.z = e[4] | (e[5] << 16); u.w = e[6] | (e[7] << 16);
  return u;
}

__device__ __forceinline__ uint32_t mask2(uint32_t v, uint32_t m, float slope) {
  float v0 = __uint_as_float(v << 16), v1 = __uint_as_float(v & 0xffff0000u);
  float m0 = __uint_as_float(m << 16), m1 = __uint_as_float(m & 0xffff0000u);
  if (!(m0 > 0.f)) v0 *= slope;
  if (!(m1 > 0.f)) v1 *= slope;
  return (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
}

// SMALLCI (Cin <= 5: the first layer of both networks): the 48 columns 0..47 hold every (ci,kd,kh)
// combination, so instead of splitting columns the four wavefronts of a workgroup split the K-steps
// of each tile and their accumulators are added in wavefront order at the end.
// DMA: the tiles go global -> LDS directly (buffer_load ... lds, 16 bytes per lane, no registers and no
// VALU in between; lanes whose unit is padding or lies outside the volume use an out-of-range offset
// and deposit zeros).  Needs whole 16-byte units (W % 8 == 0, aligned bases) and no fused mask.
template <int RBW, int NRG, int TW, int TH, bool MASKED, bool SMALLCI, bool DMA>
__global__ void __launch_bounds__(SMALLCI ? 256 : 192 * NRG, DMA ? 3 : 1) bwd_filter_mfma_kernel(const bf16_t* __restrict__ x,
                                                                              const bf16_t* __restrict__ dz,
                                                                              const bf16_t* __restrict__ z,
                                                                              float* __restrict__ part, BfmArgs a) {
  using T = BfTile<TW, TH>;
  static_assert(!SMALLCI || NRG == 1, "row groups only in the column-split mode");
  constexpr int NW = SMALLCI ? 4 : 3 * NRG;   // NRG groups of three wavefronts, each group owns RBW row blocks
  constexpr int NT = 64 * NW;
  constexpr int CI_WG = SMALLCI ? 6 : 16;     // channels staged per workgroup
  constexpr int CO_WG = 16 * RBW * NRG;
  static_assert(!(DMA && MASKED), "the mask needs the register path");
  constexpr int XPAD = (CI_WG * T::PC + 63) / 64 * 64;     // x region rounded up to whole 64-unit DMA chunks
  constexpr int GPAD = (CO_WG * T::PG + 63) / 64 * 64;
  extern __shared__ uint4 lds[];
  uint4* xl = lds;                    // [CI_WG][3 kd][TH+2 rows][PR units]  (pitches PC, PD, PR)
  uint4* gl = lds + XPAD;             // [CO_WG][TH rows][GU units]          (pitch PG)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lc = lane & 15;
  // Workgroups that stream the SAME voxel chunk (all ci groups, all co groups) are made neighbours in
  // time and placed on the same XCD, so the tiles they share are served by that XCD's L2: the linear
  // block id is (chunk / 8, group, chunk % 8) and consecutive ids go to the 8 XCDs round-robin.
  const int ngrp = a.gy * a.gz;
  int chunk, grp;
  {
    const int b = blockIdx.x, full = (a.nchunks / 8) * 8 * ngrp;
    if (b < full) { chunk = (b / (8 * ngrp)) * 8 + b % 8; grp = (b / 8) % ngrp; }
    else { const int r = b - full, rem = a.nchunks % 8; chunk = (a.nchunks / 8) * 8 + r % rem; grp = r / rem; }
  }
  const int zi = grp % a.gz;
  const int co0 = (grp / a.gz) * CO_WG, ci0 = zi * 16;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  const int rg = SMALLCI ? 0 : wave / 3;       // row group of this wavefront
  const int cb0 = SMALLCI ? 0 : 3 * (wave % 3);  // first of this wavefront's three column blocks

  // ---- this lane's three column blocks: combination q = (cb0 + cbi)*16 + lc = ci_local*9 + kd*3 + kh
  int xb[3];
#pragma unroll
  for (int cbi = 0; cbi < 3; ++cbi) {
    int q = (cb0 + cbi) * 16 + lc;
    int cil = q / 9, kd = (q % 9) / 3, kh = q % 3;
    xb[cbi] = cil * T::PC + kd * T::PD + kh * T::PR + 1 + (T::GW == 4 ? lg : lg % T::GW) + (lg / T::GW) * T::PR;
  }
  const int ga_off = (rg * 16 * RBW + lc) * T::PG + (T::GW == 4 ? lg : (lg / T::GW) * T::GU + lg % T::GW);
  const bool edge_lo = (lg % T::GW) == 0, edge_hi = (lg % T::GW) == T::GW - 1;
  const int bp_prev = ((lane - 16) & 63) * 4, bp_next = ((lane + 16) & 63) * 4;
  const bool do_db = (SMALLCI || wave % 3 == 0) && (zi == 0);

  // ---- staging plan (tile-invariant part): which units this thread copies
  constexpr int XITEMS = CI_WG * 3 * (TH + 2) * T::XU;
  constexpr int XR = (XITEMS + NT - 1) / NT;
  constexpr int GITEMS = CO_WG * TH * T::GU;
  constexpr int GR = (GITEMS + NT - 1) / NT;
  int x_meta[XR];     // row | kd << 8 | u << 12 | cil << 20 | valid << 28
  int g_meta[GR];     // row | u << 8 | col << 16 | valid << 28
#pragma unroll
  for (int r = 0; r < XR; ++r) {
    int item = tid + r * NT;
    int u = item % T::XU;
    int q = item / T::XU;
    int row = q % (TH + 2); q /= (TH + 2);
    int kd = q % 3;
    int cil = q / 3;
    x_meta[r] = item < XITEMS ? (row | (kd << 8) | (u << 12) | (cil << 20) | ((ci0 + cil < a.cin ? 1 : 0) << 28)) : -1;
  }
#pragma unroll
  for (int r = 0; r < GR; ++r) {
    int item = tid + r * NT;
    int u = item % T::GU;
    int q = item / T::GU;
    int row = q % TH;
    int col = q / TH;
    g_meta[r] = item < GITEMS ? (row | (u << 8) | (col << 16) | ((co0 + col < a.cout ? 1 : 0) << 28)) : -1;
  }

  // ---- DMA plan: wavefront w owns the 64-unit LDS chunks w, w+NW, ...; lane l fills unit 64*chunk + l
  constexpr int NCHX = XPAD / 64, NCHG = GPAD / 64;
  constexpr int CXW = DMA ? (NCHX + NW - 1) / NW : 1, CGW = DMA ? (NCHG + NW - 1) / NW : 1;
  int dx_rel[CXW], dx_meta[CXW];    // byte offset relative to (plane p, row h0, column w0) of channel ci0; meta: row | kd<<8 | w8<<12, -1 = never valid
  int dg_rel[CGW], dg_meta[CGW];
  if (DMA) {
#pragma unroll
    for (int i = 0; i < CXW; ++i) {
      const int ul = 64 * (wave + NW * i) + lane;
      const int cil = ul / T::PC, r1 = ul % T::PC;
      const int kd = r1 / T::PD, r2 = r1 % T::PD;
      const int row = r2 / T::PR, u = r2 % T::PR;
      const bool ok = wave + NW * i < NCHX && cil < CI_WG && kd < 3 && row < TH + 2 && u < T::XU && ci0 + cil < a.cin;
      dx_meta[i] = ok ? (row | (kd << 8) | (u << 12)) : -1;
      dx_rel[i] = 2 * ((ci0 + cil) * (int)a.x.cstride + (kd - 1 + a.x.hlo) * (int)a.x.plane + (row - 1) * W + 8 * u - 8);
    }
#pragma unroll
    for (int i = 0; i < CGW; ++i) {
      const int ul = 64 * (wave + NW * i) + lane;
      const int col = ul / T::PG, r1 = ul % T::PG;
      const int row = r1 / T::GU, u = r1 % T::GU;
      const bool ok = wave + NW * i < NCHG && col < CO_WG && r1 < TH * T::GU && co0 + col < a.cout;
      dg_meta[i] = ok ? (row | (u << 12)) : -1;
      dg_rel[i] = 2 * ((co0 + col) * (int)a.g.cstride + a.g.hlo * (int)a.g.plane + row * W + 8 * u);
    }
  }

  f32x4 acc[RBW][3][3];
  f32x4 accdb[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    accdb[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cbi = 0; cbi < 3; ++cbi)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) acc[rb][cbi][kw] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint4 ones_u = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_u);

  // tile coordinates are decoded once and then advanced incrementally (no divisions in the loop)
  const int t_begin = chunk * a.tiles_per_chunk;
  const int t_end = min(t_begin + a.tiles_per_chunk, (int)a.ntiles);
  int tw, th, p, n;
  {
    int r = t_begin;
    tw = r % a.tiles_w; r /= a.tiles_w;
    th = r % a.tiles_h; r /= a.tiles_h;
    p = r % D;
    n = r / D;
  }
  for (int tile = t_begin; tile < t_end; ++tile, ++tw) {
    if (tw == a.tiles_w) { tw = 0; ++th; }
    if (th == a.tiles_h) { th = 0; ++p; }
    if (p == D) { p = 0; ++n; }
    const int w0 = tw * TW, h0 = th * TH;

    if (DMA) {
      __syncthreads();   // everyone is done reading the previous tile
      const h3d_i32x4 rs_x = bf_rsrc(x + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
      const h3d_i32x4 rs_g = bf_rsrc(dz + n * a.g.nstride, (uint32_t)a.g.nstride * 2);
      const int tx = 2 * (p * (int)a.x.plane + h0 * W + w0), tg = 2 * (p * (int)a.g.plane + h0 * W + w0);
#pragma unroll
      for (int i = 0; i < CXW; ++i) {
        const int m = dx_meta[i];
        const int row = m & 0xff, kd = (m >> 8) & 0xf, w = w0 + 8 * ((m >> 12) & 0xff) - 8;
        const int h = h0 + row - 1;
        const int64_t gq = a.x.doff + p + kd - 1;
        const bool ok = m >= 0 && h >= 0 && h < H && gq >= 0 && gq < a.x.dglob && w >= 0 && w + 8 <= W;
        if (wave + NW * i < NCHX)
          dma16(rs_x, xl + 64 * (wave + NW * i), ok ? tx + dx_rel[i] : BF_OOB);
      }
#pragma unroll
      for (int i = 0; i < CGW; ++i) {
        const int m = dg_meta[i];
        const int row = m & 0xff, w = w0 + 8 * ((m >> 12) & 0xff);
        const bool ok = m >= 0 && h0 + row < H && w + 8 <= W;
        if (wave + NW * i < NCHG)
          dma16(rs_g, gl + 64 * (wave + NW * i), ok ? tg + dg_rel[i] : BF_OOB);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    } else {
    // ---- global -> registers for this tile (issued before the barrier so they overlap the
    //      other wavefronts' last K-steps), then registers -> LDS
    uint4 xv[XR], gv[GR], mvv[MASKED ? GR : 1];
    const bf16_t* xt = x + n * a.x.nstride + (int64_t)(p + a.x.hlo - 1) * a.x.plane + (int64_t)(h0 - 1) * W + w0;
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      const int m = x_meta[i];
      const int row = m & 0xff, kd = (m >> 8) & 0xf, u = (m >> 12) & 0xff, cil = (m >> 20) & 0xff;
      const int h = h0 + row - 1;
      const int64_t gq = a.x.doff + p + kd - 1;
      const bool ok = m >= 0 && (m >> 28) && h >= 0 && h < H && gq >= 0 && gq < a.x.dglob;
      xv[i] = load_unit(xt + (int64_t)(ci0 + cil) * a.x.cstride + (int64_t)kd * a.x.plane + row * W, w0 + 8 * u - 8, W, ok,
                        a.vec_ok, w0);
    }
    const bf16_t* gt = dz + n * a.g.nstride + (int64_t)(p + a.g.hlo) * a.g.plane + (int64_t)h0 * W + w0;
    const bf16_t* zt = MASKED ? z + n * a.z.nstride + (int64_t)(p + a.z.hlo) * a.z.plane + (int64_t)h0 * W + w0 : nullptr;
#pragma unroll
    for (int i = 0; i < GR; ++i) {
      const int m = g_meta[i];
      const int row = m & 0xff, u = (m >> 8) & 0xff, col = (m >> 16) & 0xfff;
      const bool ok = m >= 0 && (m >> 28) && h0 + row < H;
      gv[i] = load_unit(gt + (int64_t)(co0 + col) * a.g.cstride + row * W, w0 + 8 * u, W, ok, a.vec_ok, w0);
      if (MASKED) mvv[i] = load_unit(zt + (int64_t)(co0 + col) * a.z.cstride + row * W, w0 + 8 * u, W, ok, a.vec_ok, w0);
    }
    __syncthreads();   // everyone is done reading the previous tile
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      const int m = x_meta[i];
      if (m >= 0) xl[((m >> 20) & 0xff) * T::PC + ((m >> 8) & 0xf) * T::PD + (m & 0xff) * T::PR + ((m >> 12) & 0xff)] = xv[i];
    }
#pragma unroll
    for (int i = 0; i < GR; ++i) {
      const int m = g_meta[i];
      if (m < 0) continue;
      uint4 v = gv[i];
      if (MASKED) {
        v.x = mask2(v.x, mvv[i].x, a.mask_slope); v.y = mask2(v.y, mvv[i].y, a.mask_slope);
        v.z = mask2(v.z, mvv[i].z, a.mask_slope); v.w = mask2(v.w, mvv[i].w, a.mask_slope);
      }
      gl[((m >> 16) & 0xfff) * T::PG + (m & 0xff) * T::GU + ((m >> 8) & 0xff)] = v;
    }
    __syncthreads();

    }

    // ---- K-steps of 32 voxels
#pragma unroll
    for (int ks = 0; ks < T::KSTEPS; ++ks) {
      if (SMALLCI && (ks % NW) != wave) continue;
      // position of this K-step inside the tile: row (first row of the step) and unit offset
      const int row = T::GW == 4 ? ks / T::KS_PER_ROW : ks * T::RPK;
      const int uo = T::GW == 4 ? (ks % T::KS_PER_ROW) * 4 : 0;
      bf16x8 A[RBW];
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) A[rb] = __builtin_bit_cast(bf16x8, gl[rb * 16 * T::PG + ga_off + row * T::GU + uo]);
      if (do_db) {
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) accdb[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[rb], ones, accdb[rb], 0, 0, 0);
      }
#pragma unroll
      for (int cbi = 0; cbi < 3; ++cbi) {
        const int ua = xb[cbi] + row * T::PR + uo;
        const uint4 blk = xl[ua];
        uint32_t pv = __builtin_amdgcn_ds_bpermute(bp_prev, blk.w);
        uint32_t nx = __builtin_amdgcn_ds_bpermute(bp_next, blk.x);
        const uint32_t* xw = reinterpret_cast<const uint32_t*>(xl);
        if (edge_lo) pv = xw[(ua - 1) * 4 + 3];
        if (edge_hi) nx = xw[(ua + 1) * 4];
        const uint32_t s0 = __builtin_amdgcn_alignbit(blk.x, pv, 16);
        const uint32_t s1 = __builtin_amdgcn_alignbit(blk.y, blk.x, 16);
        const uint32_t s2 = __builtin_amdgcn_alignbit(blk.z, blk.y, 16);
        const uint32_t s3 = __builtin_amdgcn_alignbit(blk.w, blk.z, 16);
        const uint32_t s4 = __builtin_amdgcn_alignbit(nx, blk.w, 16);
        const uint4 f0 = {s0, s1, s2, s3}, f2 = {s1, s2, s3, s4};
        const bf16x8 B0 = __builtin_bit_cast(bf16x8, f0), B1 = __builtin_bit_cast(bf16x8, blk), B2 = __builtin_bit_cast(bf16x8, f2);
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
          acc[rb][cbi][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[rb], B0, acc[rb][cbi][0], 0, 0, 0);
          acc[rb][cbi][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[rb], B1, acc[rb][cbi][1], 0, 0, 0);
          acc[rb][cbi][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[rb], B2, acc[rb][cbi][2], 0, 0, 0);
        }
      }
    }
  }

  if (SMALLCI) {
    // add the four wavefronts' accumulators in wavefront order (fixed, so the result is reproducible)
    f32x4* red = reinterpret_cast<f32x4*>(lds);     // [3][64] slots, reused for every accumulator
    auto wave_sum = [&](f32x4& v) {
      __syncthreads();
      if (wave > 0) red[(wave - 1) * 64 + lane] = v;
      __syncthreads();
      if (wave == 0) v = ((v + red[lane]) + red[64 + lane]) + red[128 + lane];
    };
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      wave_sum(accdb[rb]);
#pragma unroll
      for (int cbi = 0; cbi < 3; ++cbi)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wave_sum(acc[rb][cbi][kw]);
    }
    if (wave > 0) return;
  }

  // ---- partial tile -> workspace [chunk][cout][cin][27] (+ [chunk][cout] for the bias partial behind it)
  float* pw = part + (int64_t)chunk * a.cout * a.cin * 27;
#pragma unroll
  for (int cbi = 0; cbi < 3; ++cbi) {
    const int q = (cb0 + cbi) * 16 + lc;
    const int ci = ci0 + q / 9, kdkh = q % 9;
    if (ci >= a.cin) continue;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + (rg * RBW + rb) * 16 + 4 * lg + rr;
        if (co < a.cout) {
          float* o = pw + ((int64_t)co * a.cin + ci) * 27 + kdkh * 3;
          o[0] = acc[rb][cbi][0][rr];
          o[1] = acc[rb][cbi][1][rr];
          o[2] = acc[rb][cbi][2][rr];
        }
      }
  }
  if (do_db && lc == 0) {
    float* pb = part + (int64_t)a.nchunks * a.cout * a.cin * 27 + (int64_t)chunk * a.cout;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + (rg * RBW + rb) * 16 + 4 * lg + rr;
        if (co < a.cout) pb[co] = accdb[rb][rr];
      }
  }
}

// ---------------------------------------------------------------------------------------------------
// Row-rolling variant for the wide layers (W >= 32, whole 16-byte units, no fused mask).
//
// Same GEMM, different split of the 27 taps: a column block is 16 input channels of ONE kd plane (a
// wavefront per kd), and the kh taps are not columns but ROWS: the operand built from x row r pairs
// with g row r - kh.  So one aligned 16-byte LDS read of an x row segment (plus its two edge dwords)
// feeds 9 x RBW MFMAs (3 kh x 3 kw), and each g row fragment is read once and kept in registers while
// three x rows pass.  Nothing in the inner loop depends on a branch: the edge dwords of a row segment
// are read by all lanes of a column from one address (a broadcast) and travel to the lane group that
// needs them inside the same ds_bpermute that exchanges the neighbours' dwords.
//
// Tiles are walked along DEPTH first.  The x planes live in a ring of four LDS slots (plane q in slot
// q mod 4): a step in depth brings in ONE new plane, the other two are already there.  While a tile is
// being multiplied, the next tile's plane and g tile are on their way into the free slot / the other g
// buffer (buffer_load ... lds), so a tile costs one barrier and the copies overlap the MFMAs.
// A workgroup = 3 kd x CIB channel blocks x NRG row groups of wavefronts.
template <int TH>
struct RollTile {
  static constexpr int TW = 32;
  static constexpr int XU = TW / 8 + 2;            // x row: w in [w0-8, w0+TW+8)
  static constexpr int PCI = ((TH + 2) * XU) | 1;  // odd channel pitch: the 16 channels of a column block hit 16 bank groups
  static constexpr int GU = TW / 8;
  static constexpr int PG = (TH * GU) | 1;
};

template <int RBW, int NRG, int CIB, int TH>
__global__ void __launch_bounds__(192 * NRG * CIB, 3) bwd_filter_roll_kernel(const bf16_t* __restrict__ x,
                                                                           const bf16_t* __restrict__ dz,
                                                                           float* __restrict__ part, BfmArgs a) {
  using T = RollTile<TH>;
  constexpr int NW = 3 * NRG * CIB;
  constexpr int CO_WG = 16 * RBW * NRG, CI_WG = 16 * CIB;
  constexpr int SLOTP = (CI_WG * T::PCI + 63) / 64 * 64;      // one plane of the x tile, whole 64-unit copy chunks
  constexpr int GPAD = (CO_WG * T::PG + 63) / 64 * 64;
  constexpr int NCHX = SLOTP / 64, NCHG = GPAD / 64;
  constexpr int CXW = (NCHX + NW - 1) / NW, CGW = (NCHG + NW - 1) / NW;
  extern __shared__ uint4 lds[];
  uint4* xl = lds;                    // [4 slots][CI_WG][TH+2 rows][6 units]  (pitches SLOTP, PCI, XU)
  uint4* gl = lds + 4 * SLOTP;        // [2 buffers][CO_WG][TH rows][4 units]  (pitches GPAD, PG, GU)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lc = lane & 15;
  const int ngrp = a.gy * a.gz * a.wpair;
  int chunk, grp;
  {
    const int b = blockIdx.x, full = (a.nchunks / 8) * 8 * ngrp;
    if (b < full) { chunk = (b / (8 * ngrp)) * 8 + b % 8; grp = (b / 8) % ngrp; }
    else { const int r = b - full, rem = a.nchunks % 8; chunk = (a.nchunks / 8) * 8 + r % rem; grp = r / rem; }
  }
  const int par = grp % a.wpair;      // which of the two 32-column tiles of a 64-column pair
  grp /= a.wpair;
  const int zi = grp % a.gz;
  const int co0 = (grp / a.gz) * CO_WG, ci0 = zi * CI_WG;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  const int kd = wave % 3, cib = (wave / 3) % CIB, rg = wave / (3 * CIB);
  const bool edge_lo = lg == 0, edge_hi = lg == 3;
  const int bp_prev = ((lane - 16) & 63) * 4, bp_next = ((lane + 16) & 63) * 4;
  const bool do_db = kd == 0 && cib == 0 && zi == 0;
  // per-lane LDS byte offsets inside a slot / a g buffer; rows and row blocks are compile-time offsets on top
  const int xb_o = 16 * ((cib * 16 + lc) * T::PCI + 1 + lg);
  const int pe_o = 16 * ((cib * 16 + lc) * T::PCI) + 12;       // last dword of unit 0 of the row
  const int ga_o = 16 * ((rg * 16 * RBW + lc) * T::PG + lg);

  // copy plan: wavefront w fills the 64-unit chunks w, w + NW, ... of a slot (or g buffer); lane l fills unit 64 * chunk + l
  int dx_meta[CXW];    // row | u << 8 | ci << 16, -1 = padding or channel out of range
  int dg_meta[CGW];    // row | u << 8 | co << 16
#pragma unroll
  for (int i = 0; i < CXW; ++i) {
    const int ul = 64 * (wave + NW * i) + lane;
    const int cil = ul / T::PCI, r1 = ul % T::PCI;
    const int row = r1 / T::XU, u = r1 % T::XU;
    const bool ok = wave + NW * i < NCHX && cil < CI_WG && row < TH + 2 && ci0 + cil < a.cin;
    dx_meta[i] = ok ? (row | (u << 8) | ((ci0 + cil) << 16)) : -1;
  }
#pragma unroll
  for (int i = 0; i < CGW; ++i) {
    const int ul = 64 * (wave + NW * i) + lane;
    const int col = ul / T::PG, r1 = ul % T::PG;
    const int row = r1 / T::GU, u = r1 % T::GU;
    const bool ok = wave + NW * i < NCHG && col < CO_WG && row < TH && co0 + col < a.cout;
    dg_meta[i] = ok ? (row | (u << 8) | ((co0 + col) << 16)) : -1;
  }

  auto roll_dma = [&](h3d_i32x4 rs, uint4* dst, int voff) {
    if (NRG * CIB > 1) dma16(rs, dst, voff);
    else dma16_visible(rs, dst, voff);
  };
  // plane q (relative to the slab's first owned plane) of sample n, rows h0-1.., columns w0-8.. -> slot q mod 4
  auto load_plane = [&](int n, int q, int h0, int w0) {
    const h3d_i32x4 rs = bf_rsrc(x + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
    const int64_t gq = a.x.doff + q;
    const bool plane_ok = gq >= 0 && gq < a.x.dglob;
    const int t0 = (q + a.x.hlo) * (int)a.x.plane + (h0 - 1) * W + w0 - 8;
    uint4* dst = xl + ((q + 4) & 3) * SLOTP;
#pragma unroll
    for (int i = 0; i < CXW; ++i) {
      int m = dx_meta[i];
      // opaque to the optimiser: otherwise every field of every plan entry is unpacked once, kept in a
      // register of its own across the tile loop, and the accumulators are spilled to make room
      asm volatile("" : "+v"(m));
      const int row = m & 0xff, u8 = 8 * ((m >> 8) & 0xff), ci = m >> 16;
      const int w = w0 + u8 - 8, h = h0 + row - 1;
      const bool ok = m >= 0 && plane_ok && h >= 0 && h < H && w >= 0 && w + 8 <= W;
      if (wave + NW * i < NCHX)
        roll_dma(rs, dst + 64 * (wave + NW * i), ok ? 2 * (t0 + ci * (int)a.x.cstride + row * W + u8) : BF_OOB);
    }
  };
  auto load_g = [&](int n, int q, int h0, int w0, int buf) {
    const h3d_i32x4 rs = bf_rsrc(dz + n * a.g.nstride, (uint32_t)a.g.nstride * 2);
    const int t0 = (q + a.g.hlo) * (int)a.g.plane + h0 * W + w0;
    uint4* dst = gl + buf * GPAD;
#pragma unroll
    for (int i = 0; i < CGW; ++i) {
      int m = dg_meta[i];
      asm volatile("" : "+v"(m));
      const int row = m & 0xff, u8 = 8 * ((m >> 8) & 0xff), co = m >> 16;
      const bool ok = m >= 0 && h0 + row < H && w0 + u8 + 8 <= W;
      if (wave + NW * i < NCHG)
        roll_dma(rs, dst + 64 * (wave + NW * i), ok ? 2 * (t0 + co * (int)a.g.cstride + row * W + u8) : BF_OOB);
    }
  };

  f32x4 acc[RBW][3][3];   // [row block][kh][kw]
  f32x4 accdb[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    accdb[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) acc[rb][kh][kw] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint4 ones_u = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_u);

  // tile order: depth fastest, then columns, rows, samples
  const int t_begin = chunk * a.tiles_per_chunk;
  const int t_end = min(t_begin + a.tiles_per_chunk, (int)a.ntiles);
  int tw, th, p, n;
  {
    int r = t_begin;
    p = r % D; r /= D;
    tw = r % a.tiles_w; r /= a.tiles_w;
    th = r % a.tiles_h;
    n = r / a.tiles_h;
  }
  if (t_begin < t_end) {
    load_plane(n, p - 1, th * TH, (tw * a.wpair + par) * T::TW);
    load_plane(n, p, th * TH, (tw * a.wpair + par) * T::TW);
    load_plane(n, p + 1, th * TH, (tw * a.wpair + par) * T::TW);
    load_g(n, p, th * TH, (tw * a.wpair + par) * T::TW, 0);
  }
  int buf = 0;
  for (int tile = t_begin; tile < t_end; ++tile) {
    // this tile's copies have landed (each wavefront waits for its own, the barrier collects them all),
    // and everyone is done with the previous tile, whose g buffer and oldest plane are now free
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int tw2 = tw, th2 = th, p2 = p + 1, n2 = n;
    if (p2 == D) { p2 = 0; ++tw2; }
    if (tw2 == a.tiles_w) { tw2 = 0; ++th2; }
    if (th2 == a.tiles_h) { th2 = 0; ++n2; }
    const bool has_next = tile + 1 < t_end;
    const bool jump = has_next && p2 == 0;      // the next tile starts a new column of tiles: none of its planes is here
    if (has_next) {
      load_g(n2, p2, th2 * TH, (tw2 * a.wpair + par) * T::TW, buf ^ 1);
      if (!jump) load_plane(n2, p2 + 1, th2 * TH, (tw2 * a.wpair + par) * T::TW);
    }

    const char* xs = reinterpret_cast<const char*>(xl) + 16 * SLOTP * ((p + kd + 3) & 3);   // plane p + kd - 1
    const char* xb_p = xs + xb_o;
    const char* pe_p = xs + pe_o;
    const char* ga_p = reinterpret_cast<const char*>(gl) + 16 * GPAD * buf + ga_o;

    // Row loop.  Per x row r: B(r) = {row r shifted by -1, 0, +1}; MFMA groups in the order kh = 2, 1, 0
    // (g rows r-2, r-1, r), so the register slot of g row r-2 is free after the first group and takes g
    // row r+1, which is first needed at the END of the next iteration.  The LDS reads of x row r+1 are
    // issued at the top of iteration r; its cross-lane exchange sits between the first two MFMA groups.
    uint4 blk[2];
    uint32_t pe, ne, pv, nx;
    bf16x8 A[3][RBW];
    bf16x8 B0, B1, B2;
    auto read_x = [&](int r) {      // x row r: aligned block + the two edge dwords of the row segment
      const int off = 16 * T::XU * r;
      blk[r & 1] = *reinterpret_cast<const uint4*>(xb_p + off);
      pe = *reinterpret_cast<const uint32_t*>(pe_p + off);
      ne = *reinterpret_cast<const uint32_t*>(pe_p + off + 16 * (T::XU - 1) - 12);
    };
    auto read_g = [&](int r) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb)
        A[r % 3][rb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ga_p + 16 * (rb * 16 * T::PG + r * T::GU)));
    };
    auto exchange = [&](int r) {
      // The dword before / after this lane's block.  Lane group 3's last dword is wanted by nobody (its
      // "next" group is group 0 by wrap-around), so it hands the segment's low edge dword to group 0
      // instead; likewise group 0 hands the high edge dword to group 3.
      pv = __builtin_amdgcn_ds_bpermute(bp_prev, edge_hi ? pe : blk[r & 1].w);
      nx = __builtin_amdgcn_ds_bpermute(bp_next, edge_lo ? ne : blk[r & 1].x);
    };
    auto build_B = [&](int r) {
      const uint4 b = blk[r & 1];
      const uint32_t s0 = __builtin_amdgcn_alignbit(b.x, pv, 16);
      const uint32_t s1 = __builtin_amdgcn_alignbit(b.y, b.x, 16);
      const uint32_t s2 = __builtin_amdgcn_alignbit(b.z, b.y, 16);
      const uint32_t s3 = __builtin_amdgcn_alignbit(b.w, b.z, 16);
      const uint32_t s4 = __builtin_amdgcn_alignbit(nx, b.w, 16);
      const uint4 f0 = {s0, s1, s2, s3}, f2 = {s1, s2, s3, s4};
      B0 = __builtin_bit_cast(bf16x8, f0); B1 = __builtin_bit_cast(bf16x8, b); B2 = __builtin_bit_cast(bf16x8, f2);
    };
    auto mfma_group = [&](int r, int kh) {   // x row r meets g row r - kh under tap row kh
      const int gr = r - kh;
      if (gr < 0 || gr >= TH) return;
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        acc[rb][kh][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B0, acc[rb][kh][0], 0, 0, 0);
        acc[rb][kh][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B1, acc[rb][kh][1], 0, 0, 0);
        acc[rb][kh][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B2, acc[rb][kh][2], 0, 0, 0);
      }
    };
    read_x(0);
    read_g(0);
    exchange(0);
#pragma unroll
    for (int r = 0; r < TH + 2; ++r) {
      build_B(r);
      if (r + 1 < TH + 2) read_x(r + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(r, 2);
      __builtin_amdgcn_sched_barrier(0);
      if (r + 1 < TH) read_g(r + 1);
      if (r + 1 < TH + 2) exchange(r + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(r, 1);
      mfma_group(r, 0);
      if (r < TH && do_db) {
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) accdb[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[r % 3][rb], ones, accdb[rb], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    if (jump) {
      __syncthreads();    // three of the four slots are about to be rewritten: everyone must be done with this tile
      load_plane(n2, -1, th2 * TH, (tw2 * a.wpair + par) * T::TW);
      load_plane(n2, 0, th2 * TH, (tw2 * a.wpair + par) * T::TW);
      load_plane(n2, 1, th2 * TH, (tw2 * a.wpair + par) * T::TW);
    }
    tw = tw2; th = th2; p = p2; n = n2;
    buf ^= 1;
  }

  // ---- partial tile -> workspace [chunk][cout][cin][27] (+ [chunk][cout] for the bias partial behind it)
  const int pchunk = chunk * a.wpair + par;
  float* pw = part + (int64_t)pchunk * a.cout * a.cin * 27;
  const int ci = ci0 + cib * 16 + lc;
  if (ci < a.cin) {
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + (rg * RBW + rb) * 16 + 4 * lg + rr;
        if (co < a.cout) {
          float* o = pw + ((int64_t)co * a.cin + ci) * 27 + kd * 9;
#pragma unroll
          for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) o[kh * 3 + kw] = acc[rb][kh][kw][rr];
        }
      }
  }
  if (do_db && lc == 0) {
    float* pb = part + (int64_t)a.npart * a.cout * a.cin * 27 + (int64_t)pchunk * a.cout;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + (rg * RBW + rb) * 16 + 4 * lg + rr;
        if (co < a.cout) pb[co] = accdb[rb][rr];
      }
  }
}

// Row-rolling kernel for the first layer of a network (Cin <= 4).  One column block holds every
// (ci, kd) combination (column = 3 ci + kd), so a single wavefront covers all 27 taps: kd through the
// lane's plane slot, kh through the rolling g rows, kw through the shifted operands.  The NW wavefronts
// of a workgroup share the staged tile and split its rows into bands of RB (each band reads RB + 2 x
// rows); their accumulators are added in wavefront order at the end.  Pitches: channel pitch = 1 and
// slot pitch = 4 (mod 16), so the 16 columns of a block read 16 distinct bank groups.
// NSEG segments of 32 columns per row: with NSEG = 2 a row of the tile is a whole 128-byte line of the tensors,
// so no line is fetched by two workgroups at two different times.
template <int TH, int NSEG>
struct RollSmallTile {
  static constexpr int TW = 32 * NSEG, XU = 4 * NSEG + 2, GU = 4 * NSEG;
  static constexpr int PCI = cmod_ge((TH + 2) * XU, 1);
  static constexpr int NCHX = (4 * PCI + 63) / 64;            // 64-unit copy chunks of one plane (4 channels)
  static constexpr int SLOTP = cmod_ge(NCHX * 64, 4);
  static constexpr int PG = (TH * GU) | 1;
};

template <int RBW, int NW, int RB, int NSEG>
__global__ void __launch_bounds__(64 * NW, NW == 4 ? 4 : 2) bwd_filter_roll_small_kernel(const bf16_t* __restrict__ x,
                                                                         const bf16_t* __restrict__ dz,
                                                                         float* __restrict__ part, BfmArgs a) {
  constexpr int TH = NW * RB;
  using T = RollSmallTile<TH, NSEG>;
  constexpr int CO_WG = 16 * RBW;
  constexpr int SLOTP = T::SLOTP, NCHX = T::NCHX;
  constexpr int CXW = (NCHX + NW - 1) / NW;
  extern __shared__ uint4 lds[];
  uint4* xl = lds;                    // [4 slots][4 ci][TH+2 rows][6 units]  (pitches SLOTP, PCI, XU)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lc = lane & 15;
  int chunk, grp;
  {
    const int ngrp = a.gy;
    const int b = blockIdx.x, full = (a.nchunks / 8) * 8 * ngrp;
    if (b < full) { chunk = (b / (8 * ngrp)) * 8 + b % 8; grp = (b / 8) % ngrp; }
    else { const int r = b - full, rem = a.nchunks % 8; chunk = (a.nchunks / 8) * 8 + r % rem; grp = r / rem; }
  }
  const int co0 = grp * CO_WG;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  const int cil = lc / 3, kdl = lc % 3;
  const bool col_ok = cil < a.cin;              // columns beyond 3 Cin compute on channel 0 and are dropped
  const bool edge_lo = lg == 0, edge_hi = lg == 3;
  const int bp_prev = ((lane - 16) & 63) * 4, bp_next = ((lane + 16) & 63) * 4;
  const int row0 = wave * RB;                   // this wavefront's band of the tile
  const int xb_o = 16 * ((col_ok ? cil : 0) * T::PCI + row0 * T::XU + 1 + lg);
  const int pe_o = 16 * ((col_ok ? cil : 0) * T::PCI + row0 * T::XU) + 12;

  int dx_meta[CXW];    // row | u << 8 | ci << 16, -1 = padding or channel out of range
#pragma unroll
  for (int i = 0; i < CXW; ++i) {
    const int ul = 64 * (wave + NW * i) + lane;
    const int ci = ul / T::PCI, r1 = ul % T::PCI;
    const int row = r1 / T::XU, u = r1 % T::XU;
    const bool ok = wave + NW * i < NCHX && ci < 4 && row < TH + 2 && ci < a.cin;
    dx_meta[i] = ok ? (row | (u << 8) | (ci << 16)) : -1;
  }
  auto load_plane = [&](int n, int q, int h0, int w0) {
    const h3d_i32x4 rs = bf_rsrc(x + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
    const int64_t gq = a.x.doff + q;
    const bool plane_ok = gq >= 0 && gq < a.x.dglob;
    const int t0 = (q + a.x.hlo) * (int)a.x.plane + (h0 - 1) * W + w0 - 8;
    uint4* dst = xl + ((q + 4) & 3) * SLOTP;
#pragma unroll
    for (int i = 0; i < CXW; ++i) {
      int m = dx_meta[i];
      asm volatile("" : "+v"(m));     // keeps the unpacked fields from being hoisted into registers of their own
      const int row = m & 0xff, u8 = 8 * ((m >> 8) & 0xff), ci = m >> 16;
      const int w = w0 + u8 - 8, h = h0 + row - 1;
      const bool ok = m >= 0 && plane_ok && h >= 0 && h < H && w >= 0 && w + 8 <= W;
      if (wave + NW * i < NCHX)
        dma16(rs, dst + 64 * (wave + NW * i), ok ? 2 * (t0 + ci * (int)a.x.cstride + row * W + u8) : BF_OOB);
    }
  };
  // The g rows of a wavefront's band are used by that wavefront alone, and 8 consecutive voxels of one channel are
  // 16 contiguous bytes: they go straight from global memory into the A-operand registers (lane (lc, lg): channel
  // co0 + 16 rb + lc, voxels 8 lg .. 8 lg + 7 of the 32-column segment), one tile ahead, without touching LDS.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto load_g = [&](u32x4 (&G)[RB][NSEG][RBW], int n, int q, int h0, int w0) {
    const __amdgpu_buffer_rsrc_t rs = bf_rsrc_reg(dz + n * a.g.nstride, (uint32_t)a.g.nstride * 2);
    const int t0 = (q + a.g.hlo) * (int)a.g.plane + (h0 + row0) * W + w0 + 8 * lg;
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
      for (int seg = 0; seg < NSEG; ++seg)
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
          const int co = co0 + 16 * rb + lc;
          const bool ok = co < a.cout && h0 + row0 + r < H && w0 + 32 * seg + 8 * lg + 8 <= W;
          G[r][seg][rb] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? 2 * (t0 + co * (int)a.g.cstride + r * W + 32 * seg) : BF_OOB, 0, 0);
        }
  };

  f32x4 acc[RBW][3][3];   // [row block][kh][kw]
  f32x4 accdb[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    accdb[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) acc[rb][kh][kw] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint4 ones_u = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_u);

  const int t_begin = chunk * a.tiles_per_chunk;
  const int t_end = min(t_begin + a.tiles_per_chunk, (int)a.ntiles);
  int tw, th, p, n;
  {
    int r = t_begin;
    p = r % D; r /= D;
    tw = r % a.tiles_w; r /= a.tiles_w;
    th = r % a.tiles_h;
    n = r / a.tiles_h;
  }
  u32x4 G0[RB][NSEG][RBW], G1[RB][NSEG][RBW];     // this tile's g rows and the next tile's
  if (t_begin < t_end) {
    load_plane(n, p - 1, th * TH, tw * T::TW);
    load_plane(n, p, th * TH, tw * T::TW);
    load_plane(n, p + 1, th * TH, tw * T::TW);
    load_g(G0, n, p, th * TH, tw * T::TW);
  }
  auto tile_step = [&](u32x4 (&Gc)[RB][NSEG][RBW], u32x4 (&Gn)[RB][NSEG][RBW], int tile) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int tw2 = tw, th2 = th, p2 = p + 1, n2 = n;
    if (p2 == D) { p2 = 0; ++tw2; }
    if (tw2 == a.tiles_w) { tw2 = 0; ++th2; }
    if (th2 == a.tiles_h) { th2 = 0; ++n2; }
    const bool has_next = tile + 1 < t_end;
    const bool jump = has_next && p2 == 0;
    if (has_next) {
      load_g(Gn, n2, p2, th2 * TH, tw2 * T::TW);
      if (!jump) load_plane(n2, p2 + 1, th2 * TH, tw2 * T::TW);
    }

    const char* xs = reinterpret_cast<const char*>(xl) + 16 * SLOTP * ((p + kdl + 3) & 3);   // this lane's plane p + kd - 1
#pragma unroll
    for (int seg = 0; seg < NSEG; ++seg) {
    const char* xb_p = xs + xb_o + 64 * seg;
    const char* pe_p = xs + pe_o + 64 * seg;

    uint4 blk[2];
    uint32_t pe, ne, pv, nx;
    bf16x8 A[3][RBW];
    bf16x8 B0, B1, B2;
    auto read_x = [&](int r) {
      const int off = 16 * T::XU * r;
      blk[r & 1] = *reinterpret_cast<const uint4*>(xb_p + off);
      pe = *reinterpret_cast<const uint32_t*>(pe_p + off);
      ne = *reinterpret_cast<const uint32_t*>(pe_p + off + 16 * 5 - 12);
    };
    auto read_g = [&](int r) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) A[r % 3][rb] = __builtin_bit_cast(bf16x8, Gc[r][seg][rb]);
    };
    auto exchange = [&](int r) {
      pv = __builtin_amdgcn_ds_bpermute(bp_prev, edge_hi ? pe : blk[r & 1].w);
      nx = __builtin_amdgcn_ds_bpermute(bp_next, edge_lo ? ne : blk[r & 1].x);
    };
    auto build_B = [&](int r) {
      const uint4 b = blk[r & 1];
      const uint32_t s0 = __builtin_amdgcn_alignbit(b.x, pv, 16);
      const uint32_t s1 = __builtin_amdgcn_alignbit(b.y, b.x, 16);
      const uint32_t s2 = __builtin_amdgcn_alignbit(b.z, b.y, 16);
      const uint32_t s3 = __builtin_amdgcn_alignbit(b.w, b.z, 16);
      const uint32_t s4 = __builtin_amdgcn_alignbit(nx, b.w, 16);
      const uint4 f0 = {s0, s1, s2, s3}, f2 = {s1, s2, s3, s4};
      B0 = __builtin_bit_cast(bf16x8, f0); B1 = __builtin_bit_cast(bf16x8, b); B2 = __builtin_bit_cast(bf16x8, f2);
    };
    auto mfma_group = [&](int r, int kh) {
      const int gr = r - kh;
      if (gr < 0 || gr >= RB) return;
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        acc[rb][kh][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B0, acc[rb][kh][0], 0, 0, 0);
        acc[rb][kh][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B1, acc[rb][kh][1], 0, 0, 0);
        acc[rb][kh][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[gr % 3][rb], B2, acc[rb][kh][2], 0, 0, 0);
      }
    };
    read_x(0);
    read_g(0);
    exchange(0);
#pragma unroll
    for (int r = 0; r < RB + 2; ++r) {
      build_B(r);
      if (r + 1 < RB + 2) read_x(r + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(r, 2);
      __builtin_amdgcn_sched_barrier(0);
      if (r + 1 < RB) read_g(r + 1);
      if (r + 1 < RB + 2) exchange(r + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(r, 1);
      mfma_group(r, 0);
      if (r < RB) {
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) accdb[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[r % 3][rb], ones, accdb[rb], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    }

    if (jump) {
      __syncthreads();
      load_plane(n2, -1, th2 * TH, tw2 * T::TW);
      load_plane(n2, 0, th2 * TH, tw2 * T::TW);
      load_plane(n2, 1, th2 * TH, tw2 * T::TW);
    }
    tw = tw2; th = th2; p = p2; n = n2;
  };
  for (int tile = t_begin; tile < t_end; tile += 2) {
    tile_step(G0, G1, tile);
    if (tile + 1 < t_end) tile_step(G1, G0, tile + 1);
  }

  // add the wavefronts' accumulators in wavefront order (fixed, so the result is reproducible)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  f32x4* red = reinterpret_cast<f32x4*>(lds);     // [NW-1][64] slots, reused for every accumulator
  auto wave_sum = [&](f32x4& v) {
    __syncthreads();
    if (wave > 0) red[(wave - 1) * 64 + lane] = v;
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int wv = 0; wv < NW - 1; ++wv) v = v + red[wv * 64 + lane];
    }
  };
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    wave_sum(accdb[rb]);
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) wave_sum(acc[rb][kh][kw]);
  }
  if (wave > 0) return;

  float* pw = part + (int64_t)chunk * a.cout * a.cin * 27;
  if (col_ok && lc < 15) {
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + rb * 16 + 4 * lg + rr;
        if (co < a.cout) {
          float* o = pw + ((int64_t)co * a.cin + cil) * 27 + kdl * 9;
#pragma unroll
          for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) o[kh * 3 + kw] = acc[rb][kh][kw][rr];
        }
      }
  }
  if (lc == 0) {
    float* pb = part + (int64_t)a.nchunks * a.cout * a.cin * 27 + (int64_t)chunk * a.cout;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int co = co0 + rb * 16 + 4 * lg + rr;
        if (co < a.cout) pb[co] = accdb[rb][rr];
      }
  }
}

// Second stage: out[i] = sum over chunks of part[chunk][i] in a FIXED order.  A block takes 16
// consecutive outputs; G thread groups (16, or 64 when there are many chunks) each add every G-th chunk in
// increasing order, then the G group sums are added in group order.  (dw and the bias partials share the kernel: the bias
// partials are stored behind the dw partials.)
template <int G>
__global__ void __launch_bounds__(16 * G) bfm_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                            float* __restrict__ db, int64_t nw, int cout, int nchunks) {
  __shared__ float red[G][17];
  const int o = threadIdx.x & 15, cg = threadIdx.x >> 4;
  const int64_t i = (int64_t)blockIdx.x * 16 + o;
  const int64_t nout = nw + cout;
  float s = 0.f;
  if (i < nout) {
    const bool is_w = i < nw;
    const float* base = is_w ? part + i : part + (int64_t)nchunks * nw + (i - nw);
    const int64_t stride = is_w ? nw : cout;
    int c = cg;
    for (; c + 7 * G < nchunks; c += 8 * G) {      // eight loads in flight, added in increasing chunk order
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = base[(int64_t)(c + u * G) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nchunks; c += G) s += base[(int64_t)c * stride];
  }
  red[cg][o] = s;
  __syncthreads();
  if (cg == 0 && i < nout) {
    float t = red[0][o];
#pragma unroll
    for (int k = 1; k < G; ++k) t += red[k][o];
    if (i < nw) dw[i] = t;
    else if (db) db[i - nw] = t;
  }
}

// The same sum, same order, four weights per thread (nw a multiple of 4, 16-byte-aligned partials): 16 lanes read
// 256 contiguous bytes of a chunk row instead of 64.
__global__ void __launch_bounds__(256) bfm_reduce4_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                          float* __restrict__ db, int64_t nw, int cout, int nchunks) {
  __shared__ float4 red[16][17];
  const int o = threadIdx.x & 15, cg = threadIdx.x >> 4;
  const int64_t nq = nw / 4, nblk_w = (nq + 15) / 16;
  if ((int64_t)blockIdx.x < nblk_w) {
    const int64_t q = (int64_t)blockIdx.x * 16 + o;
    float4 s = {0.f, 0.f, 0.f, 0.f};
    if (q < nq) {
      for (int c = cg; c < nchunks; c += 16) {
        const float4 v = reinterpret_cast<const float4*>(part + (int64_t)c * nw)[q];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
    }
    red[cg][o] = s;
    __syncthreads();
    if (cg == 0 && q < nq) {
      float4 t = red[0][o];
#pragma unroll
      for (int k = 1; k < 16; ++k) { t.x += red[k][o].x; t.y += red[k][o].y; t.z += red[k][o].z; t.w += red[k][o].w; }
      reinterpret_cast<float4*>(dw)[q] = t;
    }
  } else {
    __shared__ float redb[16][17];
    const int64_t i = ((int64_t)blockIdx.x - nblk_w) * 16 + o;
    float s = 0.f;
    if (i < cout) {
      const float* base = part + (int64_t)nchunks * nw + i;
      for (int c = cg; c < nchunks; c += 16) s += base[(int64_t)c * cout];
    }
    redb[cg][o] = s;
    __syncthreads();
    if (cg == 0 && i < cout && db) {
      float t = redb[0][o];
#pragma unroll
      for (int k = 1; k < 16; ++k) t += redb[k][o];
      db[i] = t;
    }
  }
}

// Same sum for many outputs and few chunks (the late, channel-rich layers): one thread per output adds the chunks
// in increasing order, so every chunk row is read in whole contiguous kilobytes.
__global__ void __launch_bounds__(256) bfm_reduce_wide_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                              float* __restrict__ db, int64_t nw, int cout, int nchunks) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nw + cout) return;
  const bool is_w = i < nw;
  const float* base = is_w ? part + i : part + (int64_t)nchunks * nw + (i - nw);
  const int64_t stride = is_w ? nw : cout;
  float s = 0.f;
  int c = 0;
  for (; c + 4 <= nchunks; c += 4) {
    const float a0 = base[(int64_t)c * stride], a1 = base[(int64_t)(c + 1) * stride];
    const float a2 = base[(int64_t)(c + 2) * stride], a3 = base[(int64_t)(c + 3) * stride];
    s = (((s + a0) + a1) + a2) + a3;
  }
  for (; c < nchunks; ++c) s += base[(int64_t)c * stride];
  if (is_w) dw[i] = s;
  else if (db) db[i - nw] = s;
}

struct BfPlan {
  int tw, th, rbw, nrg, cib, wpair;
  bool smallci;
  int tiles_w, tiles_h;
  int64_t ntiles;
  int tiles_per_chunk, nchunks;
};

// The row-rolling kernel takes the wide layers with more than a handful of input channels.
static bool bf_roll_shape(const h3d_tensor* x) { return x->w >= 32 && (x->c > 5 || (x->c <= 4 && x->h >= 16)); }

static BfPlan bf_plan_mfma(const h3d_tensor* x, int cout, bool roll) {
  BfPlan p;
  p.smallci = x->c <= 5;
  p.rbw = cout <= 16 ? 1 : 2;
  p.nrg = (cout > 32 && !p.smallci) ? 2 : 1;
  p.cib = 1;
  if (roll) {
    // workgroup = 3 kd x cib channel blocks x nrg row groups of wavefronts; Cout in steps of 16 * rbw * nrg
    p.tw = 32;
    p.rbw = cout > 32 ? 2 : 1;
    p.nrg = cout > 16 ? 2 : 1;
    p.cib = x->c > 16 ? 2 : 1;
    p.th = (p.rbw == 2 && p.cib == 2 && x->h >= 48) ? 6 : 4;
    if (p.cib == 1 && cout > 16 && cout <= 32) { p.rbw = 2; p.nrg = 1; p.th = 6; }   // one 3-wavefront row group, taller tiles
    if (x->c <= 4) {    // first-layer kernel: one wavefront covers all taps, 8 wavefronts split the tile's rows
      p.smallci = false;
      // wide volumes: 16 output channels per workgroup whatever Cout is (every group reads its own channels of g once;
      // only the few input channels are read once per group), so that the 64-column form below serves them all
      p.rbw = (cout > 16 && x->w < 64) ? 2 : 1;
      p.nrg = 1;
      p.th = p.rbw == 2 ? 16 : 32;
      if (p.rbw == 1 && x->w >= 64) { p.tw = 64; p.th = 8; }     // whole 128-byte lines per tile row; 4 wavefronts, two workgroups per CU
    }
  }
  else if (x->w > 32) { p.tw = 64; p.th = 2; }
  else if (x->w > 16) { p.tw = 32; p.th = 4; }
  else { p.tw = 16; p.th = 4; }
  p.tiles_w = (int)cdiv(x->w, p.tw);
  // rolling kernel, 32-column tiles: neighbouring tiles share 128-byte lines, so they are walked as pairs by two
  // workgroups side by side (the pair index counts as a workgroup group, not as tiles)
  p.wpair = (roll && x->c > 4 && p.tiles_w >= 2) ? 2 : 1;
  p.tiles_w = (int)cdiv(p.tiles_w, p.wpair);
  p.tiles_h = (int)cdiv(x->h, p.th);
  p.ntiles = (int64_t)x->n * x->d * p.tiles_h * p.tiles_w;
  int64_t groups = cdiv(cout, 16 * p.rbw * p.nrg) * cdiv(x->c, 16 * p.cib) * p.wpair;
  // Number of voxel chunks: enough workgroups to fill 256 CUs several times over, at least 4 tiles
  // per workgroup, and partials (chunks x Cout x Cin x 27 floats) that stay small next to the tensors.
  int64_t per_chunk_bytes = std::max<int64_t>(1, (int64_t)cout * x->c * 27 * 4);
  int64_t want = std::max<int64_t>(1, 1024 / groups);
  int64_t cap_bytes = (int64_t)48 << 20;
  if (roll) {
    // the rolling kernels hold one to three workgroups per CU (LDS-bound): one round of resident workgroups,
    // which keeps the fp32 partials (written once, read once by the reduction) small next to the tensors
    int per_cu = 1;
    if (x->c > 4) per_cu = (p.cib == 2) ? 1 : (p.rbw * p.nrg == 1 ? 3 : 2);
    else if (p.tw == 64) per_cu = 2;     // two workgroups of 4 wavefronts per CU (measured: more of them only compete for the memory system)
    want = std::max<int64_t>(1, cdiv(256 * per_cu, groups));
    cap_bytes = (int64_t)96 << 20;
  }
  want = std::min<int64_t>(want, std::max<int64_t>(1, cap_bytes / per_chunk_bytes));
  want = std::min<int64_t>(want, std::max<int64_t>(1, p.ntiles / 4));
  p.tiles_per_chunk = (int)std::max<int64_t>(1, cdiv(p.ntiles, want));
  p.nchunks = (int)std::max<int64_t>(1, cdiv(p.ntiles, p.tiles_per_chunk));
  return p;
}

// the kernel on the 32x32x16 tile (bwd_filter_row32.hip)
bool row32_bf_shape(const h3d_tensor* x, const h3d_tensor* dz);
int row32_bf_nchunks(const h3d_tensor* x, const h3d_tensor* dz);
h3d_status row32_bf_partials(void* handle, const h3d_tensor* x, const h3d_tensor* dz, float* part, int* npart, hipStream_t stream);

bool mfma_bf_supported(const h3d_tensor* x, const h3d_tensor* dz) {
  if (x->dtype != H3D_BF16 || x->c < 1 || dz->c < 1) return false;
  return sample_span(x) < ((int64_t)1 << 40) && (int64_t)(x->halo_lo + x->d + x->halo_hi) * x->h * x->w < ((int64_t)1 << 30);
}

size_t mfma_bf_ws_bytes(const h3d_tensor* x, const h3d_tensor* dz) {
  // which kernel runs also depends on alignment and on the fused mask, unknown here: size for either
  int nchunks = bf_plan_mfma(x, dz->c, false).nchunks;
  if (bf_roll_shape(x)) {
    const BfPlan pr = bf_plan_mfma(x, dz->c, true);
    nchunks = std::max(nchunks, pr.nchunks * pr.wpair);
  }
  if (row32_bf_shape(x, dz)) nchunks = std::max(nchunks, row32_bf_nchunks(x, dz));
  return (size_t)nchunks * ((size_t)dz->c * x->c * 27 + dz->c) * sizeof(float);
}

template <int RBW, int NRG, int CIB, int TH>
static h3d_status bf_roll_launch(void* handle, const bf16_t* x, const bf16_t* dz, float* part, const BfmArgs& a, dim3 grid,
                                 hipStream_t stream) {
  using T = RollTile<TH>;
  // four plane slots of the x tile and two g buffers
  constexpr size_t lds_bytes = (size_t)(4 * ((16 * CIB * T::PCI + 63) / 64 * 64) + 2 * ((16 * RBW * NRG * T::PG + 63) / 64 * 64)) * 16;
  auto kern = bwd_filter_roll_kernel<RBW, NRG, CIB, TH>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d_bwd_filter: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(192 * NRG * CIB), lds_bytes, stream, x, dz, part, a);
  note_kernel(handle, "bwd_filter_roll_kernel<%d,%d,%d,%d>", RBW, NRG, CIB, TH);
  return H3D_OK;
}

template <int RBW, int NW, int RB, int NSEG>
static h3d_status bf_roll_small_launch(void* handle, const bf16_t* x, const bf16_t* dz, float* part, const BfmArgs& a, dim3 grid,
                                       hipStream_t stream) {
  using T = RollSmallTile<NW * RB, NSEG>;
  constexpr size_t lds_bytes = (size_t)4 * T::SLOTP * 16;      // four plane slots; the wavefront sums at the end reuse them
  static_assert(lds_bytes >= (size_t)(NW - 1) * 64 * 16, "room for the accumulator exchange");
  auto kern = bwd_filter_roll_small_kernel<RBW, NW, RB, NSEG>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d_bwd_filter: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(64 * NW), lds_bytes, stream, x, dz, part, a);
  note_kernel(handle, "bwd_filter_roll_small_kernel<%d,%d,%d,%d>", RBW, NW, RB, NSEG);
  return H3D_OK;
}

template <int RBW, int NRG, int TW, int TH, bool MASKED, bool SMALLCI, bool DMA>
static h3d_status bf_launch(void* handle, const bf16_t* x, const bf16_t* dz, const bf16_t* z, float* part, const BfmArgs& a,
                            dim3 grid, hipStream_t stream) {
  using T = BfTile<TW, TH>;
  constexpr size_t tile_bytes = (size_t)(((SMALLCI ? 6 : 16) * T::PC + 63) / 64 * 64 + (16 * RBW * NRG * T::PG + 63) / 64 * 64) * 16;
  constexpr size_t lds_bytes = tile_bytes < 3 * 64 * 16 ? 3 * 64 * 16 : tile_bytes;
  auto kern = bwd_filter_mfma_kernel<RBW, NRG, TW, TH, MASKED, SMALLCI, DMA>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d_bwd_filter: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(SMALLCI ? 256 : 192 * NRG), lds_bytes, stream, x, dz, z, part, a);
  note_kernel(handle, "bwd_filter_mfma_kernel<%d,%d,%d,%d,%d,%d,%d>", RBW, NRG, TW, TH, (int)MASKED, (int)SMALLCI, (int)DMA);
  return H3D_OK;
}

template <int RBW, int NRG, bool MASKED, bool SMALLCI>
static h3d_status bf_pick_tile(void* handle, const BfPlan& p, const bf16_t* x, const bf16_t* dz, const bf16_t* z, float* part,
                               const BfmArgs& a, dim3 grid, hipStream_t s) {
  if constexpr (!MASKED) {
    if (a.vec_ok && a.dma_ok) {
      if (p.tw == 64) return bf_launch<RBW, NRG, 64, 2, false, SMALLCI, true>(handle, x, dz, z, part, a, grid, s);
      if (p.tw == 32) return bf_launch<RBW, NRG, 32, 4, false, SMALLCI, true>(handle, x, dz, z, part, a, grid, s);
      return bf_launch<RBW, NRG, 16, 4, false, SMALLCI, true>(handle, x, dz, z, part, a, grid, s);
    }
  }
  if (p.tw == 64) return bf_launch<RBW, NRG, 64, 2, MASKED, SMALLCI, false>(handle, x, dz, z, part, a, grid, s);
  if (p.tw == 32) return bf_launch<RBW, NRG, 32, 4, MASKED, SMALLCI, false>(handle, x, dz, z, part, a, grid, s);
  return bf_launch<RBW, NRG, 16, 4, MASKED, SMALLCI, false>(handle, x, dz, z, part, a, grid, s);
}

template <bool MASKED>
static h3d_status bf_pick(void* handle, const BfPlan& p, const bf16_t* x, const bf16_t* dz, const bf16_t* z, float* part,
                          const BfmArgs& a, dim3 grid, hipStream_t s) {
  if (p.smallci) {
    if (p.rbw == 1) return bf_pick_tile<1, 1, MASKED, true>(handle, p, x, dz, z, part, a, grid, s);
    return bf_pick_tile<2, 1, MASKED, true>(handle, p, x, dz, z, part, a, grid, s);
  }
  if (p.rbw == 1) return bf_pick_tile<1, 1, MASKED, false>(handle, p, x, dz, z, part, a, grid, s);
  if (p.nrg == 1) return bf_pick_tile<2, 1, MASKED, false>(handle, p, x, dz, z, part, a, grid, s);
  return bf_pick_tile<2, 2, MASKED, false>(handle, p, x, dz, z, part, a, grid, s);
}

h3d_status bwd_filter_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw, float* db,
                           float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  const bool vec_ok = (x->w % 8 == 0) && ((uintptr_t)x->data % 16 == 0) && ((uintptr_t)dz->data % 16 == 0) && (!z || (uintptr_t)z->data % 16 == 0);
  const bool dma_ok = sample_span(x) * 2 < ((int64_t)1 << 31) && sample_span(dz) * 2 < ((int64_t)1 << 31);
  const bool row32 = !z && vec_ok && dma_ok && row32_bf_shape(x, dz) && sample_span(x) % 8 == 0 && sample_span(dz) % 8 == 0 &&
                     x->c_stride % 8 == 0 && dz->c_stride % 8 == 0;
  const bool roll = !row32 && !z && vec_ok && dma_ok && bf_roll_shape(x);
  BfPlan p = bf_plan_mfma(x, dz->c, roll);
  if (!ws || ws_bytes < mfma_bf_ws_bytes(x, dz)) return fail(handle, H3D_EWORKSPACE, "conv3d_bwd_filter: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d_bwd_filter: workspace must be 16-byte aligned");
  BfmArgs a;
  a.x = make_geo(x); a.g = make_geo(dz); a.z = z ? make_geo(z) : a.g;
  a.cin = x->c; a.cout = dz->c;
  a.tiles_w = p.tiles_w; a.tiles_h = p.tiles_h; a.ntiles = p.ntiles;
  a.tiles_per_chunk = p.tiles_per_chunk; a.nchunks = p.nchunks;
  a.wpair = p.wpair; a.npart = p.nchunks * p.wpair;
  a.mask_slope = mask_slope;
  a.dma_ok = dma_ok;
  a.vec_ok = vec_ok;
  int64_t gy = cdiv(a.cout, 16 * p.rbw * p.nrg), gz = cdiv(a.cin, 16 * p.cib);
  if (gy > 65535 || gz > 65535) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: too many channels");
  if (p.ntiles >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: too many tiles");
  a.gy = (int)gy; a.gz = (int)gz;
  if ((int64_t)p.nchunks * gy * gz * p.wpair >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: too many workgroups");
  dim3 grid((unsigned)((int64_t)p.nchunks * gy * gz * p.wpair));
  const bf16_t* xp = (const bf16_t*)x->data;
  const bf16_t* gp = (const bf16_t*)dz->data;
  const bf16_t* zp = z ? (const bf16_t*)z->data : nullptr;
  h3d_status st;
  if (row32) {
    st = row32_bf_partials(handle, x, dz, (float*)ws, &a.npart, stream);
  } else if (roll && x->c <= 4) {
    if (p.rbw == 2) st = bf_roll_small_launch<2, 8, 2, 1>(handle, xp, gp, (float*)ws, a, grid, stream);
    else if (p.tw == 64) st = bf_roll_small_launch<1, 4, 2, 2>(handle, xp, gp, (float*)ws, a, grid, stream);
    else st = bf_roll_small_launch<1, 8, 4, 1>(handle, xp, gp, (float*)ws, a, grid, stream);
  } else if (roll) {
    if (p.cib == 2) {
      if (p.rbw == 2 && p.th == 6) st = bf_roll_launch<2, 2, 2, 6>(handle, xp, gp, (float*)ws, a, grid, stream);
      else if (p.rbw == 2) st = bf_roll_launch<2, 2, 2, 4>(handle, xp, gp, (float*)ws, a, grid, stream);
      else if (p.nrg == 2) st = bf_roll_launch<1, 2, 2, 4>(handle, xp, gp, (float*)ws, a, grid, stream);
      else st = bf_roll_launch<1, 1, 2, 4>(handle, xp, gp, (float*)ws, a, grid, stream);
    } else {
      if (p.rbw == 2 && p.nrg == 1) st = bf_roll_launch<2, 1, 1, 6>(handle, xp, gp, (float*)ws, a, grid, stream);
      else if (p.rbw == 2) st = bf_roll_launch<2, 2, 1, 4>(handle, xp, gp, (float*)ws, a, grid, stream);
      else st = bf_roll_launch<1, 1, 1, 4>(handle, xp, gp, (float*)ws, a, grid, stream);
    }
  } else {
    st = z ? bf_pick<true>(handle, p, xp, gp, zp, (float*)ws, a, grid, stream)
           : bf_pick<false>(handle, p, xp, gp, zp, (float*)ws, a, grid, stream);
  }
  if (st != H3D_OK) return st;
  int64_t nw = (int64_t)a.cout * a.cin * 27;
  if (nw >= 65536 && a.npart <= 16)
    hipLaunchKernelGGL(bfm_reduce_wide_kernel, dim3((unsigned)cdiv(nw + a.cout, 256)), dim3(256), 0, stream, (const float*)ws, dw, db,
                       nw, a.cout, a.npart);
  else if (nw >= 32768 && nw % 4 == 0 && (uintptr_t)ws % 16 == 0 && (uintptr_t)dw % 16 == 0)     // (few weights: more, smaller workgroups)
    hipLaunchKernelGGL(bfm_reduce4_kernel, dim3((unsigned)(cdiv(nw / 4, 16) + cdiv(a.cout, 16))), dim3(256), 0, stream, (const float*)ws, dw,
                       db, nw, a.cout, a.npart);
  else if (a.npart >= 128)
    hipLaunchKernelGGL(bfm_reduce_kernel<64>, dim3((unsigned)cdiv(nw + a.cout, 16)), dim3(1024), 0, stream, (const float*)ws, dw, db, nw,
                       a.cout, a.npart);
  else
    hipLaunchKernelGGL(bfm_reduce_kernel<16>, dim3((unsigned)cdiv(nw + a.cout, 16)), dim3(256), 0, stream, (const float*)ws, dw, db, nw,
                       a.cout, a.npart);
  return launch_status(handle, "conv3d_bwd_filter_mfma");
}

}  // namespace h3d
