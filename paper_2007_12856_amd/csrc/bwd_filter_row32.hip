// Backward-filter (BF pass, Sec. III-C) on the large matrix-core tile, bf16 in / fp32 accumulate, for layers with
// many channels on both sides (Cin, Cout > 32).
//
//   dW[co][ci][kd][kh][kw] = sum over voxels v of g[co][v] * x~[ci][v + (kd,kh,kw) - 1]
//
// The contraction runs over voxels: one v_mfma_f32_32x32x16_bf16 multiplies 32 output channels (rows, operand A = g)
// by 32 input channels (columns, operand B = x shifted by the tap) over K = 16 consecutive voxels of a row; a lane
// feeds 8 consecutive voxels of one channel = 16 contiguous bytes of NCDHW, so neither tensor is transposed.
//   * The tap plane kd is a GRID dimension: a workgroup owns (64 output channels, 64 input channels, kd, a chunk of
//     the volume) and only ever pairs g plane p with x plane p + kd - 1.  Its four wavefronts (one per SIMD, two
//     workgroups per CU) take the four 32x32 channel blocks; a wavefront keeps the 9 (kh,kw) accumulator tiles of its
//     block (144 registers).
//   * The volume is walked as strips = (sample, column segment of TW voxels, band of rows, plane), plane fastest, so
//     that the three kd workgroups of a chunk (neighbours in the grid, same XCD) read the same x planes within a few
//     strips of each other.  A strip is walked down its rows in blocks of RS rows = 64 voxels per channel:
//     TW x RS = 64x1, 32x2 or 16x4.
//   * x row r meets g rows r+1, r, r-1 under kh = 0, 1, 2.  The fragments of the two older g rows stay in registers
//     and move down one place per row, so every g fragment is read from LDS once; an x row is read once as aligned
//     16-byte pieces, and the kw = 0 / 2 operands are that piece shifted by one voxel (v_alignbit), the neighbouring
//     voxel coming from the other half of the wavefront (v_permlane32_swap: lanes l and l + 32 hold consecutive
//     pieces of the same channel) or, at the ends of the segment, from one dword of the edge pieces.
//   * Blocks go global -> LDS by buffer_load ... lds (no registers, zeros for everything outside the volume, so the
//     arithmetic has no boundary cases): g blocks in a ring of four, x blocks in two buffers, loaded one step ahead
//     of their use; one workgroup barrier per block.
//   * db[co] = sum of g: plain additions of the g fragments in the kd = 1 workgroups of the first input-channel block.
// Determinism: chunks, strips and the order of the additions are fixed by the shape; every workgroup writes its
// partial tile to the workspace [chunk][cout][cin][27] (+ [chunk][cout] behind it), which the ordered reduction of
// the other backward-filter kernels adds up.
#include <stdlib.h>

#include <algorithm>
#include <type_traits>

#include "common.h"

namespace h3d {

typedef __bf16 r32_bf16x8 __attribute__((ext_vector_type(8)));
typedef float r32_f32x16 __attribute__((ext_vector_type(16)));

constexpr int R32_OOB = (int)0x80000000;   // byte offset beyond every buffer: such a lane deposits zeros

struct Row32Args {
  Geo x, g;
  int cin, cout;
  int nws, nbands, nb;        // column segments per row, row bands per plane, row blocks per band
  int nstrips;                // n * nws * nbands * d (plane fastest)
  int strips_per_chunk, nchunks;
  int gco, gci;               // channel blocks of 64
};

template <int TW, int PD>
struct Row32Tile {
  static constexpr int RS = 64 / TW;              // rows per block
  static constexpr int KS = TW / 16;              // MFMA K-steps per row
  static constexpr bool EDGE = TW > 16;           // segments narrower than the row: one extra 16-byte piece on either side
  static constexpr int GU = TW / 8, GUP = GU + 1; // 16-byte pieces per g row and channel; odd pitch (bank groups)
  static constexpr int XU = GU + (EDGE ? 2 : 0), XUP = XU + 1;
  static constexpr int XBLK = RS * 64 * XUP;      // pieces per x block [row][channel][piece]
  static constexpr int GBLK = RS * 64 * GUP;
  static constexpr int NXI = RS * XUP, NGI = RS * GUP;   // copy instructions (64 pieces each) per block
  static constexpr int NG = 3 + PD, NX = 1 + PD;   // ring of g blocks (above, same, below + in flight), x buffers
  static constexpr size_t LDS_BYTES = (size_t)(NX * XBLK + NG * GBLK) * 16;
};

__device__ __forceinline__ float r32_sum8(uint4 v) {
  float s = __uint_as_float(v.x << 16) + __uint_as_float(v.x & 0xffff0000u);
  s += __uint_as_float(v.y << 16); s += __uint_as_float(v.y & 0xffff0000u);
  s += __uint_as_float(v.z << 16); s += __uint_as_float(v.z & 0xffff0000u);
  s += __uint_as_float(v.w << 16); s += __uint_as_float(v.w & 0xffff0000u);
  return s;
}

template <int TW, int PD>
__global__ void __launch_bounds__(256, 2) bwd_filter_row32_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dz,
                                                                  float* __restrict__ part, Row32Args a) {
  using T = Row32Tile<TW, PD>;
  constexpr int RS = T::RS, KS = T::KS, GUP = T::GUP, XUP = T::XUP, NG = T::NG, NX = T::NX;
  constexpr int EDGE = T::EDGE ? 1 : 0;
  constexpr int NXW = (T::NXI + 3) / 4, NGW = (T::NGI + 3) / 4;
  extern __shared__ uint4 lds[];
  uint4* xl = lds;                     // [NX buffers][RS rows][64 ci][XUP pieces]
  uint4* gl = lds + NX * T::XBLK;      // [NG ring slots][RS rows][64 co][GUP pieces]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, lc = lane & 31;
  const int rb = wave & 1, cb = wave >> 1;
  const int ngrp = a.gco * a.gci * 3;
  int chunk, grp;
  {
    // the workgroups of eight consecutive chunks are dealt round-robin to the eight XCDs, the channel blocks and tap
    // planes of one chunk following each other on the same XCD: they read the same g and x at about the same time
    const int b = blockIdx.x, full = (a.nchunks / 8) * 8 * ngrp;
    if (b < full) { chunk = (b / (8 * ngrp)) * 8 + b % 8; grp = (b / 8) % ngrp; }
    else { const int r = b - full, rem = a.nchunks % 8; chunk = (a.nchunks / 8) * 8 + r % rem; grp = r / rem; }
  }
  const int kd = grp % 3, zci = (grp / 3) % a.gci, zco = grp / (3 * a.gci);
  const int co0 = zco * 64, ci0 = zci * 64;
  const int W = a.x.w, H = a.x.h, D = a.x.d;
  const bool do_db = kd == 1 && zci == 0 && cb == 0;

  // Copy plan: wavefront w issues the instructions w, w + 4, ... of a block; lane l of instruction k fills piece
  // 64 k + l = [row k / pitch][channel][piece].  Per lane and instruction: the byte offset of (channel, piece) inside a
  // row run, or an offset beyond every buffer for padding pieces, channels and columns outside the tensor (fixed per
  // strip, rebuilt when the column segment may have changed); per step only the row's offset is added.
  int xv[NXW], gv[NGW];
  auto plan = [&](int col0) {
#pragma unroll
    for (int j = 0; j < NXW; ++j) {
      const int k = wave + 4 * j, rem = 64 * (k % XUP) + lane;
      const int c = rem / XUP, u = rem % XUP, wcol = col0 + 8 * (u - EDGE);
      const bool ok = u < T::XU && ci0 + c < a.cin && wcol >= 0 && wcol + 8 <= W;
      xv[j] = ok ? 2 * ((ci0 + c) * (int)a.x.cstride + 8 * u) : R32_OOB;
    }
#pragma unroll
    for (int j = 0; j < NGW; ++j) {
      const int k = wave + 4 * j, rem = 64 * (k % GUP) + lane;
      const int c = rem / GUP, u = rem % GUP;
      const bool ok = u < T::GU && co0 + c < a.cout && col0 + 8 * u + 8 <= W;
      gv[j] = ok ? 2 * ((co0 + c) * (int)a.g.cstride + 8 * u) : R32_OOB;
    }
  };
  h3d_i32x4 rs_g = {0, 0, 0, 0}, rs_x = {0, 0, 0, 0};
  const uint32_t xl_addr = lds_addr_of(xl), gl_addr = lds_addr_of(gl);
  // planes p whose x plane p + kd - 1 lies inside the volume: the others are neither loaded nor multiplied
  const int p_lo = (int)max((int64_t)0, 1 - kd - a.x.doff), p_hi = (int)min((int64_t)D, a.x.dglob - a.x.doff - kd + 1);
  auto planes_ok = [&](int p) { return p >= p_lo && p < p_hi; };

  // Loads of one pipeline step = position sig of a strip: g block sig - 1 (rows g_row ..) into ring slot gslot, x
  // block sig - 2 (rows x_row ..) into buffer xslot.  Every step issues the same number of instructions per wavefront
  // (steps without an x block deposit zeros), so that a wait for "all but the newest steps" is a constant count.
  // Row offsets advance by RS rows per step; rows outside [0, H) and x blocks before the band deposit zeros.
  int g_row = 0, x_row = 0, g_goff = 0, x_goff = 0, plan_key = -1;   // rows and global byte offsets of the next blocks
  bool x_plane_ok = false;
  auto strip_start = [&](int n, int ws, int band, int p) {
    const int hb0 = band * a.nb * RS, col0 = ws * TW;
    if (n * a.nws + ws != plan_key) {     // planes and bands change fastest: the plan is rebuilt once in many strips
      plan_key = n * a.nws + ws;
      plan(col0);
      rs_g = lds_dma_rsrc(dz + (int64_t)n * a.g.nstride, (uint32_t)a.g.nstride * 2);
      rs_x = lds_dma_rsrc(x + (int64_t)n * a.x.nstride, (uint32_t)a.x.nstride * 2);
    }
    g_row = hb0 - RS;
    x_row = hb0 - 2 * RS;
    g_goff = 2 * ((p + a.g.hlo) * (int)a.g.plane + g_row * W + col0);
    x_goff = 2 * ((p + kd - 1 + a.x.hlo) * (int)a.x.plane + x_row * W + col0 - 8 * EDGE);
    x_plane_ok = planes_ok(p);
  };
  auto issue = [&](int sig, int gslot, int xslot) {
    {
      const uint32_t dst = gl_addr + gslot * (T::GBLK * 16);
#pragma unroll
      for (int j = 0; j < NGW; ++j) {
        const int k = wave + 4 * j;
        if (k < T::NGI) {
          const int i = RS == 1 ? 0 : k / GUP;
          const int inv = (!x_plane_ok || (unsigned)(g_row + i) >= (unsigned)H) ? R32_OOB : 0;     // wave-uniform: the whole row lies outside
          lds_dma16(rs_g, dst + 1024 * k, (gv[j] + (g_goff + 2 * i * W)) | inv);
        }
      }
    }
    {
      const uint32_t dst = xl_addr + xslot * (T::XBLK * 16);
      const bool blk_ok = x_plane_ok && sig >= 2;
#pragma unroll
      for (int j = 0; j < NXW; ++j) {
        const int k = wave + 4 * j;
        if (k < T::NXI) {
          const int i = RS == 1 ? 0 : k / XUP;
          const int inv = (!blk_ok || x_row + i >= H) ? R32_OOB : 0;
          lds_dma16(rs_x, dst + 1024 * k, (xv[j] + (x_goff + 2 * i * W)) | inv);
        }
      }
    }
    g_row += RS; x_row += RS;
    g_goff += 2 * RS * W; x_goff += 2 * RS * W;
  };

  r32_f32x16 acc[3][3];     // [kh][kw]
#pragma unroll
  for (int kh = 0; kh < 3; ++kh)
#pragma unroll
    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[kh][kw][r] = 0.f;
  float dbacc = 0.f;
  // g row fragments in three register sets whose roles (row above, same row, row below the x row being multiplied)
  // rotate from row to row; the step loop is unrolled three times so that the roles are compile-time constants
  uint4 A[3][KS];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) A[r][ks] = uint4{0, 0, 0, 0};

  // per-lane byte offsets inside a block
  const int a_off = 16 * ((rb * 32 + lc) * GUP + half);
  const int x_off = 16 * ((cb * 32 + lc) * XUP + EDGE + half);
  const int e_off = half ? 16 * ((cb * 32 + lc) * XUP + 1 + 2 * KS) : 16 * ((cb * 32 + lc) * XUP) + 12;
  constexpr int G_ROW = 64 * GUP * 16, X_ROW = 64 * XUP * 16;
  // channel blocks that lie outside the tensors are copied (as zeros) but not multiplied
  const bool active = co0 + rb * 32 < a.cout && ci0 + cb * 32 < a.cin;

  // x block of this step against the g blocks of the two steps before and this one (ring slots g0 = oldest .. g2)
  auto compute = [&](auto r0c, int sig, int g0, int g1, int g2, int xslot) {
    constexpr int R0 = decltype(r0c)::value;
    const char* xb = reinterpret_cast<const char*>(xl + xslot * T::XBLK);
    const char* g_prev = reinterpret_cast<const char*>(gl + g0 * T::GBLK);    // g block above this x block
    const char* g_cur = reinterpret_cast<const char*>(gl + g1 * T::GBLK);     // same rows
    const char* g_next = reinterpret_cast<const char*>(gl + g2 * T::GBLK);    // below
    if (sig == 2) {   // first block of a strip: the g rows above and at the first x row
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        A[R0 % 3][ks] = *reinterpret_cast<const uint4*>(g_prev + a_off + (RS - 1) * G_ROW + 32 * ks);
        A[(R0 + 1) % 3][ks] = *reinterpret_cast<const uint4*>(g_cur + a_off + 32 * ks);
      }
    }
#pragma unroll
    for (int i = 0; i < RS; ++i) {
      uint4 (&A_old)[KS] = A[(R0 + i) % 3];
      uint4 (&A_mid)[KS] = A[(R0 + i + 1) % 3];
      uint4 (&A_new)[KS] = A[(R0 + i + 2) % 3];
      const char* gsrc = (i + 1 < RS) ? g_cur + (i + 1) * G_ROW : g_next;
      uint4 bx[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bx[ks] = *reinterpret_cast<const uint4*>(xb + x_off + i * X_ROW + 32 * ks);
        A_new[ks] = *reinterpret_cast<const uint4*>(gsrc + a_off + 32 * ks);
      }
      uint32_t edge = 0;
      if (EDGE) edge = *reinterpret_cast<const uint32_t*>(xb + e_off + i * X_ROW);
      // voxel before / after each lane's piece: from the partner lane in the other half of the wavefront, from the
      // neighbouring K-step's piece, or from the edge pieces of the segment
      uint32_t pv[KS], nx[KS];
      uint32_t pv_lo[KS], nx_hi[KS];
      pv_lo[0] = edge; nx_hi[KS - 1] = edge;
#pragma unroll
      for (int ks = 1; ks < KS; ++ks) {
        const auto r = __builtin_amdgcn_permlane32_swap(bx[ks - 1].w, bx[ks].x, false, false);
        nx_hi[ks - 1] = r[0]; pv_lo[ks] = r[1];
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const auto r = __builtin_amdgcn_permlane32_swap(bx[ks].x, bx[ks].w, false, false);
        pv[ks] = half ? r[0] : pv_lo[ks];
        nx[ks] = half ? nx_hi[ks] : r[1];
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 b = bx[ks];
        const uint32_t s0 = __builtin_amdgcn_alignbit(b.x, pv[ks], 16);
        const uint32_t s1 = __builtin_amdgcn_alignbit(b.y, b.x, 16);
        const uint32_t s2 = __builtin_amdgcn_alignbit(b.z, b.y, 16);
        const uint32_t s3 = __builtin_amdgcn_alignbit(b.w, b.z, 16);
        const uint32_t s4 = __builtin_amdgcn_alignbit(nx[ks], b.w, 16);
        const uint4 f0 = {s0, s1, s2, s3}, f2 = {s1, s2, s3, s4};
        const r32_bf16x8 B0 = __builtin_bit_cast(r32_bf16x8, f0), B1 = __builtin_bit_cast(r32_bf16x8, b),
                         B2 = __builtin_bit_cast(r32_bf16x8, f2);
        const r32_bf16x8 A0 = __builtin_bit_cast(r32_bf16x8, A_new[ks]), A1 = __builtin_bit_cast(r32_bf16x8, A_mid[ks]),
                         A2 = __builtin_bit_cast(r32_bf16x8, A_old[ks]);
        acc[2][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, B0, acc[2][0], 0, 0, 0);
        acc[2][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, B1, acc[2][1], 0, 0, 0);
        acc[2][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, B2, acc[2][2], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, B0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, B1, acc[1][1], 0, 0, 0);
        acc[1][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, B2, acc[1][2], 0, 0, 0);
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0, B0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0, B1, acc[0][1], 0, 0, 0);
        acc[0][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0, B2, acc[0][2], 0, 0, 0);
      }
      if (do_db) {     // once per row, so that the row's products stay one basic block for the scheduler
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dbacc += r32_sum8(A_mid[ks]);
      }
    }
  };

  const int s_begin = chunk * a.strips_per_chunk;
  const int s_end = min(s_begin + a.strips_per_chunk, a.nstrips);
  const int nsig = a.nb + 2;
  const int total = (s_end - s_begin) * nsig;
  int Ln, Lws, Lband, Lp, Lsig = 0;      // where the loads are: PD steps ahead of the arithmetic
  {
    int r = s_begin;
    Lp = r % D; r /= D;
    Lband = r % a.nbands; r /= a.nbands;
    Lws = r % a.nws;
    Ln = r / a.nws;
  }
  int Cp = Lp, Csig = 0;                  // where the arithmetic is
  int Lg = 0, Lx = 0;                     // ring positions of the next loads
  int Cg = 0, Cx = 0;                     // ring positions of this step's g block (the newest of the three) and x block
  auto load_next = [&]() {
    if (Lsig == 0) strip_start(Ln, Lws, Lband, Lp);
    issue(Lsig, Lg, Lx);
    if (++Lg == NG) Lg = 0;
    if (++Lx == NX) Lx = 0;
    if (++Lsig == nsig) {
      Lsig = 0;
      if (++Lp == D) {
        Lp = 0;
        if (++Lband == a.nbands) {
          Lband = 0;
          if (++Lws == a.nws) { Lws = 0; ++Ln; }
        }
      }
    }
  };
  // what a wavefront issues per step (constant, see issue()): the wait at the top of a step leaves the copies of
  // the PD - 1 newest steps in flight
  const int per_step = (T::NGI - wave + 3) / 4 + (T::NXI - wave + 3) / 4;
#pragma unroll
  for (int d = 0; d < PD; ++d)
    if (d < total) load_next();
  auto step = [&](auto r0c, int it) {
    // this step's copies have landed (each wavefront waits for its own, the barrier collects them all), and everyone
    // is done with the previous step, whose oldest g block and x block are now free
    if (PD == 1 || it + 1 >= total) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (per_step == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if (per_step == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    else if (per_step == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (it + PD < total) load_next();
    if (Csig >= 2 && active) {
      if (planes_ok(Cp))      // an x plane outside the volume contributes nothing
        compute(r0c, Csig, Cg >= 2 ? Cg - 2 : Cg - 2 + NG, Cg >= 1 ? Cg - 1 : Cg - 1 + NG, Cg, Cx);
    }
    if (++Cg == NG) Cg = 0;
    if (++Cx == NX) Cx = 0;
    if (++Csig == nsig) {
      Csig = 0;
      if (++Cp == D) Cp = 0;
    }
  };
  for (int it = 0; it < total; it += 3) {
    step(std::integral_constant<int, 0>{}, it);
    if (it + 1 < total) step(std::integral_constant<int, RS % 3>{}, it + 1);
    if (it + 2 < total) step(std::integral_constant<int, (2 * RS) % 3>{}, it + 2);
  }

  // ---- partial tile -> workspace [chunk][cout][cin][27] (+ [chunk][cout] for the bias partial behind it)
  float* pw = part + (int64_t)chunk * a.cout * a.cin * 27;
  const int ci = ci0 + cb * 32 + lc;
  if (ci < a.cin) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = co0 + rb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
      if (co < a.cout) {
        float* o = pw + ((int64_t)co * a.cin + ci) * 27 + kd * 9;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
          for (int kw = 0; kw < 3; ++kw) o[kh * 3 + kw] = acc[kh][kw][r];
      }
    }
  }
  if (do_db) {
    const uint32_t bits = __float_as_uint(dbacc);
    const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    const int co = co0 + rb * 32 + lc;
    if (half == 0 && co < a.cout)
      part[(int64_t)a.nchunks * a.cout * a.cin * 27 + (int64_t)chunk * a.cout + co] = dbacc + __uint_as_float(r[1]);
  }
}

// ---- host side -----------------------------------------------------------------------------------------------------

// Shapes the kernel takes: both channel counts above 32 (a 32-channel side would leave half of the wavefronts without
// work), rows of at least 16 voxels.  The caller adds: no fused mask, W a multiple of 8, 16-byte-aligned tensors, samples
// within 31-bit byte offsets.
struct Row32Plan {
  int tw, nb, nws, nbands, nstrips, strips_per_chunk, nchunks, gco, gci;
};

static Row32Plan row32_plan(const h3d_tensor* x, const h3d_tensor* dz);

bool row32_bf_shape(const h3d_tensor* x, const h3d_tensor* dz) {
  if (!(x->c > 32 && dz->c > 32 && x->w >= 16 && x->n > 0 && x->d > 0 && x->h > 0 &&
        (int64_t)x->n * x->d * x->h * x->w < ((int64_t)1 << 31)))
    return false;
  // small volumes with few channel blocks: a round of resident workgroups would get less than two strips each, and
  // their partial tiles would outweigh the tensors; the kernels with smaller workgroup tiles take those
  // (H3D_BF_ROW32=1 in the environment lifts this limit: the parity tests reach the kernel on shapes the oracle can do)
  const char* force = getenv("H3D_BF_ROW32");
  if (force && force[0] == '1') return true;
  const Row32Plan p = row32_plan(x, dz);
  return p.nstrips >= 2 * std::max(1, 512 / (p.gco * p.gci * 3));
}

static Row32Plan row32_plan(const h3d_tensor* x, const h3d_tensor* dz) {
  Row32Plan p;
  p.tw = x->w >= 48 ? 64 : (x->w > 16 ? 32 : 16);
  const int rs = 64 / p.tw;
  p.nb = (int)std::min<int64_t>(16 / rs, cdiv(x->h, rs));      // bands of 16 rows (8 to 64 measured alike)
  p.nbands = (int)cdiv(x->h, p.nb * rs);
  p.nws = (int)cdiv(x->w, p.tw);
  p.nstrips = (int)((int64_t)x->n * p.nws * p.nbands * x->d);
  p.gco = (int)cdiv(dz->c, 64);
  p.gci = (int)cdiv(x->c, 64);
  // one round of resident workgroups (two per CU); the fp32 partials (chunks x Cout x Cin x 27), written once and read
  // once by the reduction, are kept under 88 MB
  const int64_t groups = (int64_t)p.gco * p.gci * 3;
  const int64_t per_chunk = ((int64_t)dz->c * x->c * 27 + dz->c) * 4;
  int64_t want = std::max<int64_t>(1, 512 / groups);
  want = std::min<int64_t>(want, std::max<int64_t>(1, ((int64_t)88 << 20) / per_chunk));
  want = std::min<int64_t>(want, p.nstrips);
  p.strips_per_chunk = (int)cdiv(p.nstrips, want);
  p.nchunks = (int)cdiv(p.nstrips, p.strips_per_chunk);
  return p;
}

int row32_bf_nchunks(const h3d_tensor* x, const h3d_tensor* dz) { return row32_plan(x, dz).nchunks; }

template <int TW, int PD>
static h3d_status row32_launch(void* handle, const bf16_t* x, const bf16_t* dz, float* part, const Row32Args& a, dim3 grid,
                               hipStream_t stream) {
  using T = Row32Tile<TW, PD>;
  auto kern = bwd_filter_row32_kernel<TW, PD>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES) != hipSuccess)
      return fail(handle, H3D_EHIP, "conv3d_bwd_filter: cannot set the dynamic LDS size to %zu bytes", T::LDS_BYTES);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), T::LDS_BYTES, stream, x, dz, part, a);
  note_kernel(handle, "bwd_filter_row32_kernel<%d,%d>", TW, PD);
  return H3D_OK;
}

// Partial sums of every chunk into `part`; *npart receives the number of chunks for the ordered reduction.
h3d_status row32_bf_partials(void* handle, const h3d_tensor* x, const h3d_tensor* dz, float* part, int* npart, hipStream_t stream) {
  const Row32Plan p = row32_plan(x, dz);
  Row32Args a;
  a.x = make_geo(x); a.g = make_geo(dz);
  a.cin = x->c; a.cout = dz->c;
  a.nws = p.nws; a.nbands = p.nbands; a.nb = p.nb; a.nstrips = p.nstrips;
  a.strips_per_chunk = p.strips_per_chunk; a.nchunks = p.nchunks;
  a.gco = p.gco; a.gci = p.gci;
  const int64_t nwg = (int64_t)p.nchunks * p.gco * p.gci * 3;
  if (nwg >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: too many workgroups");
  const dim3 grid((unsigned)nwg);
  const bf16_t* xp = (const bf16_t*)x->data;
  const bf16_t* gp = (const bf16_t*)dz->data;
  *npart = p.nchunks;
  if (p.tw == 64) return row32_launch<64, 1>(handle, xp, gp, part, a, grid, stream);
  if (p.tw == 32) return row32_launch<32, 1>(handle, xp, gp, part, a, grid, stream);
  return row32_launch<16, 1>(handle, xp, gp, part, a, grid, stream);
}

}  // namespace h3d
