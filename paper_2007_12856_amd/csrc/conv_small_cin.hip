// Forward 3x3x3 convolution for the FIRST layer of both networks: Cin <= 4 input channels
// (4 redshift channels of the CosmoFlow cubes, 1 CT channel of the U-Net), Cout <= 32, bf16.
//
// With so few input channels the layer is bound by HBM (40 bytes per output voxel against 3456
// flops for 4 -> 16), so the kernel is built around the data path, not the matrix cores:
//   * the haloed input tile is staged in LDS channel-interleaved, 8 bytes per voxel (4 bf16
//     channels), from 16-byte loads along W;
//   * the contraction index is (tap, ci): K = 27*4 = 108, padded to 128 = four
//     v_mfma_f32_16x16x32_bf16 steps.  A lane's 16-byte B operand is TWO taps of one voxel, fetched
//     with two 8-byte LDS reads at per-lane tap offsets; the four lane groups of a wavefront cover
//     8 taps per step.  Output channels are the MFMA rows; the packed weights (16 x 128 per row
//     block) stay in registers for the whole kernel;
//   * the input patches are the A operand and the weights the B operand, so an accumulator holds FOUR
//     consecutive voxels of one output channel per lane: bias, activation and bf16 packing stay in the
//     lane (one bias value, packed conversions), and the row (64 voxels x Cout) goes through a per-wavefront
//     LDS patch as 8-byte pieces so that every lane stores 16 contiguous bytes along W: whole 128-byte
//     lines per channel row.
// Bias, (leaky-)ReLU and the zeroing of output planes beyond the global volume are fused.
#include <algorithm>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace c4 {
constexpr int TD = 4, TH = 4, TW = 64;
constexpr int XW = TW + 16;                 // staged row: w in [w0-8, w0+TW+8)
constexpr int PRV = XW + 2;                 // row pitch in voxels (8 bytes each)
constexpr int PDV = (TH + 2) * PRV + 6;     // plane pitch in voxels
constexpr int XS_VOX = (TD + 2) * PDV;
constexpr int OTP = TW + 8;                 // epilogue transpose pitch (bf16 elements)
}  // namespace c4

// wA: [rb][m][lane][8] bf16: row co = 16*rb + lane%16; element e of lane group g = lane/16 in step m is
// tap slot s = 2*(4m+g) + e/4, channel e%4 (zero for s >= 27, ci >= cin, co >= cout)
__global__ void pack_w_c4_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wA, int cin, int cout, int nrb) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= nrb * 4 * 512) return;
  int e = i & 7, lane = (i >> 3) & 63, m = (i >> 9) & 3, rb = i >> 11;
  int co = rb * 16 + (lane & 15), s = 2 * (4 * m + (lane >> 4)) + (e >> 2), ci = e & 3;
  bf16_t v = 0;
  if (co < cout && s < 27 && ci < cin) v = w[((int64_t)co * cin + ci) * 27 + s];
  wA[i] = v;
}

struct C4Args {
  Geo in, out;
  int cin, cout;
  int tiles_w, tiles_h, tiles_d;
  float out_slope;
  int vec_ok;
  // fused 2x2x2 average pooling (POOL kernels): pooled output, optional sign mask (one bit per unpooled voxel, 8 voxels
  // of a row per byte, rows packed [n][c][plane][h][w/8]); `out` may then be NULL (the unpooled tensor is not stored)
  Geo yp;
  bf16_t* ypool;
  uint8_t* mask;
};

template <int RB, bool POOL>
__global__ void __launch_bounds__(256) conv3d_fwd_c4_kernel(const bf16_t* __restrict__ in, const uint4* __restrict__ wA,
                                                            const float* __restrict__ bias, bf16_t* __restrict__ out, C4Args a) {
  using namespace c4;
  __shared__ uint2 xs[XS_VOX];
  __shared__ __attribute__((aligned(16))) bf16_t ot[4][16 * RB][OTP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lj = lane & 15;
  // consecutive workgroup ids go to different XCDs (each with its own L2): XCD x takes the depth slabs x, x + 8, ...
  // whole, so that the tiles of a slab, which share halo rows and columns, meet in one L2 (neighbouring slabs, in
  // different XCDs, still fetch the two shared planes twice: spreading every XCD over the whole volume keeps its
  // requests spread over the memory channels, which one contiguous run per XCD does not)
  const int per_slab = a.tiles_w * a.tiles_h, nslab = (int)gridDim.x / per_slab;
  int t = blockIdx.x;
  if (nslab % 8 == 0) {
    const int x = t % 8, i = t / 8;
    t = ((i / per_slab) * 8 + x) * per_slab + i % per_slab;
  }
  const int tw = t % a.tiles_w; t /= a.tiles_w;
  const int th = t % a.tiles_h; t /= a.tiles_h;
  const int td = t % a.tiles_d;
  const int n = t / a.tiles_d;
  const int w0 = tw * TW, h0 = th * TH, ps0 = td * TD;
  const int W = a.in.w, H = a.in.h;

  // ---- weights: registers for the whole kernel
  bf16x8 A[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int m = 0; m < 4; ++m) A[rb][m] = __builtin_bit_cast(bf16x8, wA[(rb * 4 + m) * 64 + lane]);

  // ---- per-lane tap offsets (in voxels) of the two taps this lane group feeds in each step
  int offA[4], offB[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    int s0 = 2 * (4 * m + lg), s1 = s0 + 1;
    offA[m] = s0 < 27 ? (s0 / 9) * PDV + ((s0 % 9) / 3) * PRV + s0 % 3 : 0;
    offB[m] = s1 < 27 ? (s1 / 9) * PDV + ((s1 % 9) / 3) * PRV + s1 % 3 : 0;
  }

  // ---- stage the input tile: items = (plane, row, group of 8 w), 4 channels each
  const bf16_t* in_n = in + n * a.in.nstride;
  constexpr int NGRP = XW / 8;
  constexpr int NITEMS = (TD + 2) * (TH + 2) * NGRP;
  auto transpose_store = [&](const uint4 (&c)[4], int dz, int hy, int grp) {
    uint4* dst = reinterpret_cast<uint4*>(&xs[dz * PDV + hy * PRV + 8 * grp]);
    const uint32_t c0[4] = {c[0].x, c[0].y, c[0].z, c[0].w}, c1[4] = {c[1].x, c[1].y, c[1].z, c[1].w};
    const uint32_t c2[4] = {c[2].x, c[2].y, c[2].z, c[2].w}, c3[4] = {c[3].x, c[3].y, c[3].z, c[3].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {   // voxels 2k and 2k+1 of the group
      uint4 u;
      u.x = __builtin_amdgcn_perm(c1[k], c0[k], 0x05040100);
      u.y = __builtin_amdgcn_perm(c3[k], c2[k], 0x05040100);
      u.z = __builtin_amdgcn_perm(c1[k], c0[k], 0x07060302);
      u.w = __builtin_amdgcn_perm(c3[k], c2[k], 0x07060302);
      dst[k] = u;
    }
  };
  if (a.vec_ok) {
    // whole 16-byte groups: buffer loads whose offset is pushed out of range where the group lies outside the
    // volume (they return zeros: no branches), all rounds issued before the first transpose
    constexpr int ROUNDS = (NITEMS + 255) / 256;
    constexpr int OOB = (int)0x80000000;
    // (the two halves of the pointer go through unsigned temporaries: readfirstlane returns a signed int, and a
    // sign-extended low half would overwrite the high half)
    const uint64_t pbase = reinterpret_cast<uint64_t>(in_n);
    const uint32_t p_lo = __builtin_amdgcn_readfirstlane((uint32_t)pbase), p_hi = __builtin_amdgcn_readfirstlane((uint32_t)(pbase >> 32));
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(((uint64_t)p_hi << 32) | p_lo), 0, (int)__builtin_amdgcn_readfirstlane((uint32_t)a.in.nstride * 2),
        0x00020000);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 c[ROUNDS][4];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int item = tid + 256 * r;
      const int grp = item % NGRP;
      const int q = item / NGRP;
      const int hy = q % (TH + 2), dz = q / (TH + 2);
      const int p_in = ps0 - a.out.hlo + dz - 1;
      const int64_t gq = a.in.doff + p_in;
      const int sp = p_in + a.in.hlo;
      const int h = h0 + hy - 1, w = w0 - 8 + 8 * grp;
      const bool ok = item < NITEMS && gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H && w >= 0 && w + 8 <= W;
      const int vo = ok ? 2 * (sp * (int)a.in.plane + h * W + w) : OOB;
#pragma unroll
      for (int ci = 0; ci < 4; ++ci)
        c[r][ci] = __builtin_amdgcn_raw_buffer_load_b128(rs, ci < a.cin ? vo : OOB, __builtin_amdgcn_readfirstlane(2 * ci * (int)a.in.cstride), 0);
    }
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int item = tid + 256 * r;
      if (item < NITEMS) {
        const int grp = item % NGRP;
        const int q = item / NGRP;
        const uint4 cc[4] = {uint4{c[r][0][0], c[r][0][1], c[r][0][2], c[r][0][3]}, uint4{c[r][1][0], c[r][1][1], c[r][1][2], c[r][1][3]},
                             uint4{c[r][2][0], c[r][2][1], c[r][2][2], c[r][2][3]}, uint4{c[r][3][0], c[r][3][1], c[r][3][2], c[r][3][3]}};
        transpose_store(cc, q / (TH + 2), q % (TH + 2), grp);
      }
    }
  } else {
    for (int item = tid; item < NITEMS; item += 256) {
      const int grp = item % NGRP;
      int q = item / NGRP;
      const int hy = q % (TH + 2), dz = q / (TH + 2);
      const int p_in = ps0 - a.out.hlo + dz - 1;
      const int64_t gq = a.in.doff + p_in;
      const int sp = p_in + a.in.hlo;
      const int h = h0 + hy - 1, w = w0 - 8 + 8 * grp;
      const bool row_ok = gq >= 0 && gq < a.in.dglob && sp >= 0 && sp < a.in.ds && h >= 0 && h < H;
      uint4 c[4];
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        c[ci] = uint4{0, 0, 0, 0};
        if (row_ok && ci < a.cin) {
          const bf16_t* p = in_n + (int64_t)ci * a.in.cstride + (int64_t)sp * a.in.plane + (int64_t)h * W + w;
          uint32_t e[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) e[i] = (w + i >= 0 && w + i < W) ? p[i] : 0;
          c[ci] = uint4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
        }
      }
      transpose_store(c, dz, hy, grp);
    }
  }
  __syncthreads();

  // ---- this wavefront's share of the tile, one output row (64 voxels) at a time: a depth plane and its four rows;
  //      with pooling, a PAIR of planes and a pair of rows, so that every 2x2x2 window is summed inside one lane
  float bv[RB];      // this lane's output channel of row block rb: 16 rb + lj
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) bv[rb] = (bias && rb * 16 + lj < a.cout) ? bias[rb * 16 + lj] : 0.f;
  const bool keep_row = !POOL || out || a.mask;     // the row goes through the LDS patch only if z or the mask is stored
  float psum[RB][4][2];                              // POOL: sums over the window's planes and rows, per pooled voxel
  for (int it = 0; it < TH; ++it) {
    const int pl = POOL ? 2 * (wave >> 1) + (it >> 1) : wave;      // plane and row of the tile
    const int hl = POOL ? 2 * (wave & 1) + (it & 1) : it;
    const int ps = ps0 + pl;
    const int64_t gp = a.out.doff + ps - a.out.hlo;
    const bool inside = gp >= 0 && gp < a.out.dglob;
    const bool plane_ok = ps < a.out.ds;
    bf16_t* out_n = out ? out + n * a.out.nstride + (int64_t)ps * a.out.plane : nullptr;
    f32x4 acc[4][RB];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[vb][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int vrow = pl * PDV + hl * PRV + 7 + lj;   // tap (0,0,0) of this lane's voxel in block 0
#pragma unroll
    for (int vb = 0; vb < 4; ++vb) {
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const uint2 lo = xs[vrow + vb * 16 + offA[m]], hi = xs[vrow + vb * 16 + offB[m]];
        const uint4 b = {lo.x, lo.y, hi.x, hi.y};
        const bf16x8 B = __builtin_bit_cast(bf16x8, b);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[vb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(B, A[rb][m], acc[vb][rb], 0, 0, 0);
      }
    }
    // bias + activation: accumulator register r of block vb is voxel w0 + 16 vb + 4 lg + r of channel 16 rb + lj.
    // Transposed through ot[wave][co][w]: the patch belongs to this wavefront alone and a wavefront's LDS accesses
    // execute in order, so no barrier is needed (and none that would wait for the global stores of the previous
    // row): only the compiler must keep the 8-byte writes and 16-byte reads in order.
    asm volatile("" ::: "memory");
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int vb = 0; vb < 4; ++vb) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] = acc[vb][rb][r] + bv[rb];
          if (!(v[r] > 0.f)) v[r] *= a.out_slope;
        }
        const uint2 pk = inside ? uint2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])} : uint2{0u, 0u};
        if (keep_row) *reinterpret_cast<uint2*>(&ot[wave][rb * 16 + lj][vb * 16 + 4 * lg]) = pk;
        if (POOL) {
          // the pooling reads the values as they are stored (rounded to bf16), pairs along W first
          const float s0 = __uint_as_float(pk.x << 16) + __uint_as_float(pk.x & 0xffff0000u);
          const float s1 = __uint_as_float(pk.y << 16) + __uint_as_float(pk.y & 0xffff0000u);
          if (it) { psum[rb][vb][0] += s0; psum[rb][vb][1] += s1; }
          else { psum[rb][vb][0] = s0; psum[rb][vb][1] = s1; }
        }
      }
    asm volatile("" ::: "memory");
    const int h = h0 + hl;
    if (keep_row && plane_ok && h < H) {
#pragma unroll
      for (int i = 0; i < 2 * RB; ++i) {
        const int u = lane + 64 * i;
        const int co = u >> 3, wu = u & 7;
        const int w = w0 + 8 * wu;
        if (co < a.cout && w < W) {
          const uint4 v = *reinterpret_cast<const uint4*>(&ot[wave][co][8 * wu]);
          if (out_n) {
            bf16_t* o = out_n + (int64_t)co * a.out.cstride + (int64_t)h * W + w;
            if (a.vec_ok && w + 8 <= W) {
              *reinterpret_cast<uint4*>(o) = v;
            } else {
              const uint32_t e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int k = 0; k < 8; ++k)
                if (w + k < W) o[k] = (bf16_t)(e[k >> 1] >> (16 * (k & 1)));
            }
          }
          if (POOL && a.mask) {
            // bit k of the byte: stored value of voxel w + k is > 0 (bf16 as a signed 16-bit integer: positive, not zero)
            const uint32_t e[4] = {v.x, v.y, v.z, v.w};
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
    if (POOL && it == TH - 1 && plane_ok && h < H) {
      // the window is complete (this was its last plane and row): scale, round, 4-byte stores of two pooled voxels
      bf16_t* yo = a.ypool + n * a.yp.nstride + (int64_t)((ps >> 1) + a.yp.hlo) * a.yp.plane + (int64_t)(h >> 1) * (W >> 1) + (w0 >> 1) + 2 * lg;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const int co = rb * 16 + lj;
#pragma unroll
        for (int vb = 0; vb < 4; ++vb)
          if (co < a.cout && w0 + 16 * vb + 4 * lg < W)
            *reinterpret_cast<uint32_t*>(yo + (int64_t)co * a.yp.cstride + 8 * vb) = pack_bf16x2(psum[rb][vb][0] * 0.125f, psum[rb][vb][1] * 0.125f);
      }
    }
  }
}

bool c4_fwd_supported(const h3d_tensor* in, const h3d_tensor* out) {
  if (in->dtype != H3D_BF16 || in->c < 1 || in->c > 4 || out->c < 1 || out->c > 32) return false;
  return sample_span(in) < ((int64_t)1 << 30);
}

size_t c4_fwd_ws_bytes(const h3d_tensor* out) { return (size_t)cdiv(out->c, 16) * 4 * 512 * sizeof(bf16_t); }

h3d_status conv3d_fwd_c4(void* handle, const h3d_tensor* in, const void* w, const float* bias, h3d_tensor* out, float out_slope,
                         void* ws, size_t ws_bytes, hipStream_t stream) {
  using namespace c4;
  C4Args a;
  a.in = make_geo(in); a.out = make_geo(out);
  a.cin = in->c; a.cout = out->c; a.out_slope = out_slope;
  if ((int64_t)out->n * a.out.ds * out->h * out->w == 0) return H3D_OK;
  const int nrb = (int)cdiv(out->c, 16);
  if (!ws || ws_bytes < c4_fwd_ws_bytes(out)) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd: workspace must be 16-byte aligned");
  a.vec_ok = (in->w % 8 == 0) && ((uintptr_t)in->data % 16 == 0) && ((uintptr_t)out->data % 16 == 0);
  a.tiles_w = (int)cdiv(out->w, TW); a.tiles_h = (int)cdiv(out->h, TH); a.tiles_d = (int)cdiv(a.out.ds, TD);
  int64_t grid = (int64_t)out->n * a.tiles_d * a.tiles_h * a.tiles_w;
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_fwd: too many workgroups");
  hipLaunchKernelGGL(pack_w_c4_kernel, dim3((unsigned)cdiv(nrb * 4 * 512, 256)), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws,
                     a.cin, a.cout, nrb);
  if (nrb == 1)
    hipLaunchKernelGGL((conv3d_fwd_c4_kernel<1, false>), dim3((unsigned)grid), dim3(256), 0, stream, (const bf16_t*)in->data,
                       (const uint4*)ws, bias, (bf16_t*)out->data, a);
  else
    hipLaunchKernelGGL((conv3d_fwd_c4_kernel<2, false>), dim3((unsigned)grid), dim3(256), 0, stream, (const bf16_t*)in->data,
                       (const uint4*)ws, bias, (bf16_t*)out->data, a);
  return launch_status(handle, "conv3d_fwd_c4");
}

// Fused forward + 2x2x2 average pooling (+ sign mask): z without halos, even extents, W a multiple of 8, 16-byte
// aligned tensors; y = the pooled tensor of the same shard (halos allowed, only its interior is written).
bool c4_fwd_pool_supported(const h3d_tensor* in, const h3d_tensor* z, const h3d_tensor* y) {
  if (!c4_fwd_supported(in, z) || y->dtype != H3D_BF16) return false;
  if (z->halo_lo || z->halo_hi || z->d % 2 || z->h % 2 || z->w % 8 || !is_packed(z) || !is_packed(y)) return false;
  if (y->n != z->n || y->c != z->c || y->d != z->d / 2 || y->h != z->h / 2 || y->w != z->w / 2) return false;
  if ((uintptr_t)in->data % 16 || (z->data && (uintptr_t)z->data % 16) || (uintptr_t)y->data % 4) return false;
  return true;
}

h3d_status conv3d_fwd_c4_pool(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, h3d_tensor* y,
                              void* mask, float out_slope, void* ws, size_t ws_bytes, hipStream_t stream) {
  using namespace c4;
  C4Args a;
  a.in = make_geo(in); a.out = make_geo(z); a.yp = make_geo(y);
  a.cin = in->c; a.cout = z->c; a.out_slope = out_slope;
  a.ypool = (bf16_t*)y->data; a.mask = (uint8_t*)mask;
  if ((int64_t)z->n * a.out.ds * z->h * z->w == 0) return H3D_OK;
  const int nrb = (int)cdiv(z->c, 16);
  if (!ws || ws_bytes < c4_fwd_ws_bytes(z)) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd_pool: workspace too small");
  if ((uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "conv3d_fwd_pool: workspace must be 16-byte aligned");
  a.vec_ok = 1;
  a.tiles_w = (int)cdiv(z->w, TW); a.tiles_h = (int)cdiv(z->h, TH); a.tiles_d = (int)cdiv(a.out.ds, TD);
  int64_t grid = (int64_t)z->n * a.tiles_d * a.tiles_h * a.tiles_w;
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "conv3d_fwd_pool: too many workgroups");
  hipLaunchKernelGGL(pack_w_c4_kernel, dim3((unsigned)cdiv(nrb * 4 * 512, 256)), dim3(256), 0, stream, (const bf16_t*)w, (bf16_t*)ws,
                     a.cin, a.cout, nrb);
  if (nrb == 1)
    hipLaunchKernelGGL((conv3d_fwd_c4_kernel<1, true>), dim3((unsigned)grid), dim3(256), 0, stream, (const bf16_t*)in->data,
                       (const uint4*)ws, bias, (bf16_t*)z->data, a);
  else
    hipLaunchKernelGGL((conv3d_fwd_c4_kernel<2, true>), dim3((unsigned)grid), dim3(256), 0, stream, (const bf16_t*)in->data,
                       (const uint4*)ws, bias, (bf16_t*)z->data, a);
  return launch_status(handle, "conv3d_fwd_c4_pool");
}

}  // namespace h3d
