// Filter gradient of the 2x2x2 stride-2 transposed convolution (the U-Net's up-sampling layer) on the
// matrix cores, bf16 in / fp32 accumulate:
//
//   dW[ci][co][a,b,c] = sum over coarse voxels v = (d,h,w) of x[ci][v] * dy[co][2d+a][2h+b][2w+c]
//
// a GEMM whose contraction runs over the coarse voxels.  With v_mfma_f32_16x16x32_bf16 a lane feeds 8
// consecutive voxels along W:
//   * rows    = input channels: the A operand is 16 contiguous bytes of x, staged through LDS
//     (buffer_load ... lds, double-buffered) because all 8 wavefronts of a workgroup need the same x tile;
//   * columns = (co, c) pairs, 8 output channels x 2 parities, for one (a,b): the B operand is every
//     second element of 32 contiguous bytes of a dy row, loaded straight from global memory (each dy
//     element is needed by exactly one wavefront) and de-interleaved with four byte-permutes;
//   * a workgroup = 8 wavefronts = 16 output channels x the four (a,b); each wavefront keeps
//     16*MRB input channels x 16 columns in accumulators;
//   * db[co] = sum dy: one extra MFMA per B fragment against an all-ones A operand.
// The voxel range is cut into chunks by shape alone; every workgroup writes its partial sums and a second
// kernel adds the chunks in order, so the result is reproducible.
#include <algorithm>

#include "common.h"

namespace h3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int DB_OOB = (int)0x80000000;
constexpr int DB_R = 4;                       // rows of 32 coarse voxels per tile
constexpr int DB_PCI = (4 * DB_R) | 1;        // LDS pitch of a channel in 16-byte units (odd: 16 channels -> 16 bank groups)
constexpr int DB_NW = 8;

struct DbfArgs {
  Geo x, y;
  int cin, cout;
  int tiles_w, tiles_h;
  int ntiles, tiles_per_chunk, nchunks;
  int gco, gci;       // groups of 16 output channels / of 16*MRB input channels
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t db_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p), hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                           (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

// global -> LDS copy issued so that the compiler does not wait for it before later LDS reads (common.h)
__device__ __forceinline__ void db_dma16(h3d_i32x4 rs, uint4* lds_dst, int voff) { lds_dma16(rs, lds_addr_of(lds_dst), voff); }

template <int MRB>
__global__ void __launch_bounds__(64 * DB_NW, 4) deconv_bf_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                     float* __restrict__ part, DbfArgs a) {
  constexpr int CI_WG = 16 * MRB;
  constexpr int XPAD = (CI_WG * DB_PCI + 63) / 64 * 64;
  constexpr int NCHX = XPAD / 64;
  constexpr int CXW = (NCHX + DB_NW - 1) / DB_NW;
  extern __shared__ uint4 lds[];      // [2 buffers][CI_WG][DB_R rows][4 units]  (pitches XPAD, DB_PCI, 4)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lg = lane >> 4, lc = lane & 15;
  // Workgroups go to the 8 XCDs round-robin by their linear index.  The gco * gci workgroups of one chunk read the same
  // x tiles (and, for gci > 1, the same dy rows): consecutive workgroups OF ONE XCD take the channel groups of one chunk,
  // so that they run side by side and all but the first find the tile in that XCD's L2.
  const int groups = a.gco * a.gci;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int grp = slot % groups, chunk = (slot / groups) * 8 + xcd;
  if (chunk >= a.nchunks) return;                         // the grid is padded to a multiple of 8 chunks
  const int co0 = (grp % a.gco) * 16, ci0 = (grp / a.gco) * CI_WG;
  const int ab = wave & 3, cob = wave >> 2;                // this wavefront: (a,b) and which 8 of the 16 output channels
  const int ta = ab >> 1, tb = ab & 1;
  const int co = co0 + cob * 8 + (lc >> 1), par = lc & 1;  // this lane's column: output channel and parity c
  const bool col_ok = co < a.cout;
  const uint32_t sel = par ? 0x07060302u : 0x05040100u;    // picks the odd / even halves of two dwords
  const int Wc = a.x.w, Hc = a.x.h, Dc = a.x.d, Wf = a.y.w;

  int dx_meta[CXW];    // row | u << 8 | ci << 16, -1 = padding or channel out of range
#pragma unroll
  for (int i = 0; i < CXW; ++i) {
    const int ul = 64 * (wave + DB_NW * i) + lane;
    const int cil = ul / DB_PCI, r1 = ul % DB_PCI;
    const bool ok = wave + DB_NW * i < NCHX && cil < CI_WG && r1 < 4 * DB_R && ci0 + cil < a.cin;
    dx_meta[i] = ok ? ((r1 >> 2) | ((r1 & 3) << 8) | ((ci0 + cil) << 16)) : -1;
  }
  auto load_x = [&](int n, int d, int h0, int w0, int buf) {
    const h3d_i32x4 rs = lds_dma_rsrc(x + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
    const int t0 = (d + a.x.hlo) * (int)a.x.plane + h0 * Wc + w0;
#pragma unroll
    for (int i = 0; i < CXW; ++i) {
      int m = dx_meta[i];
      asm volatile("" : "+v"(m));     // keeps the unpacked fields from being hoisted into registers of their own
      const int row = m & 0xff, u8 = 8 * ((m >> 8) & 0xff), ci = m >> 16;
      const bool ok = m >= 0 && h0 + row < Hc && w0 + u8 + 8 <= Wc;
      if (wave + DB_NW * i < NCHX)
        db_dma16(rs, lds + buf * XPAD + 64 * (wave + DB_NW * i), ok ? 2 * (t0 + ci * (int)a.x.cstride + row * Wc + u8) : DB_OOB);
    }
  };

  f32x4 acc[MRB];
  f32x4 accdb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int rb = 0; rb < MRB; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint4 ones_u = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_u);
  const bool do_db = ci0 == 0;

  // tile order: columns fastest, then row blocks, planes, samples
  const int t_begin = chunk * a.tiles_per_chunk;
  const int t_end = min(t_begin + a.tiles_per_chunk, a.ntiles);
  int tw, th, d, n;
  {
    int r = t_begin;
    tw = r % a.tiles_w; r /= a.tiles_w;
    th = r % a.tiles_h; r /= a.tiles_h;
    d = r % Dc;
    n = r / Dc;
  }
  if (t_begin < t_end) load_x(n, d, th * DB_R, tw * 32, 0);
  int buf = 0;
  const char* a_base = reinterpret_cast<const char*>(lds) + 16 * (lc * DB_PCI + lg);
  for (int tile = t_begin; tile < t_end; ++tile) {
    const int h0 = th * DB_R, w0 = tw * 32;
    // ---- this tile's dy fragments: 32 contiguous bytes per lane and row, straight from global memory
    const __amdgpu_buffer_rsrc_t rs_y = db_rsrc(dy + n * a.y.nstride, (uint32_t)a.y.nstride * 2);
    u32x4 braw[DB_R][2];
    {
      const int yb = co * (int)a.y.cstride + (2 * d + ta + a.y.hlo) * (int)a.y.plane + (2 * h0 + tb) * Wf + 2 * (w0 + 8 * lg);
#pragma unroll
      for (int r = 0; r < DB_R; ++r) {
        const bool ok = col_ok && h0 + r < Hc && w0 + 8 * lg + 8 <= Wc;
        const int off = ok ? 2 * (yb + 2 * r * Wf) : DB_OOB;
        braw[r][0] = __builtin_amdgcn_raw_buffer_load_b128(rs_y, off, 0, 0);
        braw[r][1] = __builtin_amdgcn_raw_buffer_load_b128(rs_y, ok ? off + 16 : DB_OOB, 0, 0);
      }
    }
    // the x tile of this step has landed (issued one step ago); everyone is done with the other buffer
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * DB_R) : "memory");
    __syncthreads();
    int tw2 = tw + 1, th2 = th, d2 = d, n2 = n;
    if (tw2 == a.tiles_w) { tw2 = 0; ++th2; }
    if (th2 == a.tiles_h) { th2 = 0; ++d2; }
    if (d2 == Dc) { d2 = 0; ++n2; }
    if (tile + 1 < t_end) load_x(n2, d2, th2 * DB_R, tw2 * 32, buf ^ 1);

    const char* ap = a_base + 16 * XPAD * buf;
#pragma unroll
    for (int r = 0; r < DB_R; ++r) {
      bf16x8 A[MRB];
#pragma unroll
      for (int rb = 0; rb < MRB; ++rb) A[rb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ap + 16 * (rb * 16 * DB_PCI + 4 * r)));
      uint4 bf;
      bf.x = __builtin_amdgcn_perm(braw[r][0][1], braw[r][0][0], sel);
      bf.y = __builtin_amdgcn_perm(braw[r][0][3], braw[r][0][2], sel);
      bf.z = __builtin_amdgcn_perm(braw[r][1][1], braw[r][1][0], sel);
      bf.w = __builtin_amdgcn_perm(braw[r][1][3], braw[r][1][2], sel);
      const bf16x8 B = __builtin_bit_cast(bf16x8, bf);
#pragma unroll
      for (int rb = 0; rb < MRB; ++rb) acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[rb], B, acc[rb], 0, 0, 0);
      if (do_db) accdb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, B, accdb, 0, 0, 0);
    }
    tw = tw2; th = th2; d = d2; n = n2;
    buf ^= 1;
  }

  // ---- partial sums -> workspace [chunk][cin][cout][8] (+ [chunk][cout][8] for the bias partial behind it)
  const int k = ab * 2 + par;
  if (col_ok) {
    float* pw = part + (int64_t)chunk * a.cin * a.cout * 8;
#pragma unroll
    for (int rb = 0; rb < MRB; ++rb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int ci = ci0 + rb * 16 + 4 * lg + rr;
        if (ci < a.cin) pw[((int64_t)ci * a.cout + co) * 8 + k] = acc[rb][rr];
      }
    if (do_db && lg == 0) {
      float* pb = part + (int64_t)a.nchunks * a.cin * a.cout * 8 + (int64_t)chunk * a.cout * 8;
      pb[co * 8 + k] = accdb[0];
    }
  }
}

// dw[i] = sum over chunks of part[chunk][i]; db[co] = sum over chunks and the 8 taps of the bias partials behind them.
// Fixed order: a block takes 16 consecutive outputs; each of its 16 thread groups adds every 16th chunk in increasing
// order (eight loads in flight), then the 16 group sums are added in group order.
__global__ void __launch_bounds__(256) deconv_bf_mfma_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                    float* __restrict__ db, int64_t nw, int cout, int nchunks) {
  constexpr int G = 16;
  __shared__ float red[G][17];
  const int o = threadIdx.x & 15, cg = threadIdx.x >> 4;
  const int64_t i = (int64_t)blockIdx.x * 16 + o;
  float s = 0.f;
  if (i < nw) {
    const float* base = part + i;
    int c = cg;
    for (; c + 7 * G < nchunks; c += 8 * G) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = base[(int64_t)(c + u * G) * nw];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nchunks; c += G) s += base[(int64_t)c * nw];
  } else if (db && i < nw + cout) {
    const float* pb = part + (int64_t)nchunks * nw + (i - nw) * 8;
    for (int c = cg; c < nchunks; c += G) {
      const float4 u0 = *reinterpret_cast<const float4*>(pb + (int64_t)c * cout * 8);
      const float4 u1 = *reinterpret_cast<const float4*>(pb + (int64_t)c * cout * 8 + 4);
      s += u0.x; s += u0.y; s += u0.z; s += u0.w; s += u1.x; s += u1.y; s += u1.z; s += u1.w;
    }
  }
  red[cg][o] = s;
  __syncthreads();
  if (cg == 0) {
    float r = red[0][o];
#pragma unroll
    for (int k = 1; k < G; ++k) r += red[k][o];
    if (i < nw) dw[i] = r;
    else if (db && i < nw + cout) db[i - nw] = r;
  }
}

struct DbfPlan {
  int mrb, tiles_w, tiles_h, ntiles, tiles_per_chunk, nchunks, gco, gci;
};

DbfPlan dbf_plan(const h3d_tensor* x, const h3d_tensor* dy) {
  DbfPlan p;
  p.mrb = x->c > 64 ? 8 : (x->c > 32 ? 4 : 2);
  p.tiles_w = (int)cdiv(x->w, 32);
  p.tiles_h = (int)cdiv(x->h, DB_R);
  p.ntiles = (int)((int64_t)x->n * x->d * p.tiles_h * p.tiles_w);
  p.gco = (int)cdiv(dy->c, 16);
  p.gci = (int)cdiv(x->c, 16 * p.mrb);
  const int64_t groups = (int64_t)p.gco * p.gci;
  const int64_t per_chunk_bytes = std::max<int64_t>(1, ((int64_t)x->c * dy->c + dy->c) * 8 * 4);
  int64_t want = std::max<int64_t>(1, 512 / groups);
  want = std::min<int64_t>(want, std::max<int64_t>(1, ((int64_t)64 << 20) / per_chunk_bytes));
  want = std::min<int64_t>(want, std::max<int64_t>(1, p.ntiles / 4));
  p.tiles_per_chunk = (int)std::max<int64_t>(1, cdiv(p.ntiles, want));
  p.nchunks = (int)std::max<int64_t>(1, cdiv(p.ntiles, p.tiles_per_chunk));
  return p;
}

template <int MRB>
h3d_status dbf_launch(void* handle, const bf16_t* x, const bf16_t* dy, float* part, const DbfArgs& a, hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)2 * ((16 * MRB * DB_PCI + 63) / 64 * 64) * 16;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(deconv_bf_mfma_kernel<MRB>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "deconv2_bwd_filter: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_set = true;
  }
  const int64_t grid = cdiv(a.nchunks, 8) * 8 * (int64_t)(a.gco * a.gci);
  if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "deconv2_bwd_filter: too many workgroups");
  hipLaunchKernelGGL((deconv_bf_mfma_kernel<MRB>), dim3((unsigned)grid), dim3(64 * DB_NW), lds_bytes, stream, x, dy, part, a);
  return H3D_OK;
}

}  // namespace

bool deconv_bf_mfma_supported(const h3d_tensor* x, const h3d_tensor* dy) {
  if (x->dtype != H3D_BF16 || x->c < 1 || dy->c < 1 || x->w % 8 != 0) return false;
  if ((uintptr_t)x->data % 16 != 0 || (uintptr_t)dy->data % 16 != 0) return false;
  const int64_t xs = (int64_t)x->c * (x->halo_lo + x->d + x->halo_hi) * x->h * x->w * 2;
  const int64_t ys = (int64_t)dy->c * (dy->halo_lo + dy->d + dy->halo_hi) * dy->h * dy->w * 2;
  const int64_t ntiles = (int64_t)x->n * x->d * cdiv(x->h, DB_R) * cdiv(x->w, 32);
  return xs < ((int64_t)1 << 31) && ys < ((int64_t)1 << 31) && ntiles < ((int64_t)1 << 30) && cdiv(dy->c, 16) * cdiv(x->c, 32) < 65536;
}

size_t deconv_bf_mfma_ws_bytes(const h3d_tensor* x, const h3d_tensor* dy) {
  const DbfPlan p = dbf_plan(x, dy);
  return (size_t)p.nchunks * ((size_t)x->c * dy->c + dy->c) * 8 * sizeof(float);
}

__global__ void deconv_zero_kernel(float* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

h3d_status deconv_bf_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dy, float* dw, float* db, void* ws, size_t ws_bytes,
                          hipStream_t stream) {
  const DbfPlan p = dbf_plan(x, dy);
  if (!ws || ws_bytes < deconv_bf_mfma_ws_bytes(x, dy)) return fail(handle, H3D_EWORKSPACE, "deconv2_bwd_filter: workspace too small");
  DbfArgs a;
  a.x = make_geo(x); a.y = make_geo(dy);
  a.cin = x->c; a.cout = dy->c;
  a.tiles_w = p.tiles_w; a.tiles_h = p.tiles_h; a.ntiles = p.ntiles;
  a.tiles_per_chunk = p.tiles_per_chunk; a.nchunks = p.nchunks;
  a.gco = p.gco; a.gci = p.gci;
  const int64_t nw = (int64_t)a.cin * a.cout * 8;
  if (p.ntiles == 0) {
    // a fill kernel, not a memset: the call may be recorded into a graph by the caller
    hipLaunchKernelGGL(deconv_zero_kernel, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, stream, dw, nw);
    if (db) hipLaunchKernelGGL(deconv_zero_kernel, dim3((unsigned)cdiv(a.cout, 256)), dim3(256), 0, stream, db, (int64_t)a.cout);
    return launch_status(handle, "deconv2_bwd_filter");
  }
  const bf16_t* xp = (const bf16_t*)x->data;
  const bf16_t* yp = (const bf16_t*)dy->data;
  h3d_status st;
  if (p.mrb == 8) st = dbf_launch<8>(handle, xp, yp, (float*)ws, a, stream);
  else if (p.mrb == 4) st = dbf_launch<4>(handle, xp, yp, (float*)ws, a, stream);
  else st = dbf_launch<2>(handle, xp, yp, (float*)ws, a, stream);
  if (st != H3D_OK) return st;
  hipLaunchKernelGGL(deconv_bf_mfma_reduce_kernel, dim3((unsigned)cdiv(nw + a.cout, 16)), dim3(256), 0, stream, (const float*)ws, dw,
                     db, nw, a.cout, a.nchunks);
  return launch_status(handle, "deconv2_bwd_filter_mfma");
}

}  // namespace h3d

// ---------------------------------------------------------------------------------------------------
// Data gradient of the transposed convolution:
//
//   dx[ci][v] = sum over co and the 8 taps k = (a,b,c) of W[ci][co][k] * dy[co][2d+a][2h+b][2w+c]
//
// a GEMM whose contraction index (co, k) needs no re-layout on either side: with
// v_mfma_f32_32x32x16_bf16 a lane feeds the 8 taps of ONE output channel — for the B operand the
// 2x2x2 block of dy above its coarse voxel (four dword loads, consecutive lanes = consecutive dwords),
// for the A operand 16 contiguous bytes of W[ci][co][0..8).  Rows = input channels, columns = 32 coarse
// voxels along W, one K-step = two output channels.  W^T sits in LDS for the whole (persistent)
// workgroup, as [co][ci] units with an odd pitch; every dy element is loaded exactly once.
namespace h3d {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int DD_NW = 8;
constexpr int DD_BATCH = 8;      // K-steps (pairs of output channels) whose dy loads are in flight together

struct DbdArgs {
  Geo x, y;          // x: coarse tensor (dx), y: fine tensor (dy)
  int cin, cout;
  int wblks;         // 32-voxel column blocks per coarse row
  int64_t ncb;       // column blocks in total
};

template <int MRB>
__global__ void __launch_bounds__(64 * DD_NW, 2) deconv_bd_mfma_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ w,
                                                                     bf16_t* __restrict__ dx, DbdArgs a) {
  constexpr int CP = (32 * MRB) | 1;          // LDS pitch of an output channel in 16-byte units
  extern __shared__ uint4 lds[];              // [cout rounded up to even][CP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int nks = (a.cout + 1) / 2;

  // ---- W[ci][co][8] -> LDS [co][ci]; rows of a padding channel are zero (their dy operand is zero too)
  {
    const uint4* wu = reinterpret_cast<const uint4*>(w);
    const int total = a.cin * a.cout;
    for (int i = tid; i < total; i += 64 * DD_NW) {
      const int ci = i / a.cout, co = i % a.cout;
      lds[co * CP + ci] = wu[i];
    }
    if (a.cout & 1)
      for (int i = tid; i < CP; i += 64 * DD_NW) lds[a.cout * CP + i] = uint4{0, 0, 0, 0};
  }
  __syncthreads();

  const int Wc = a.x.w, Hc = a.x.h, Dc = a.x.d, Wf = a.y.w;
  const char* a_base = reinterpret_cast<const char*>(lds) + 16 * (half * CP + col);
  for (int64_t cb = (int64_t)blockIdx.x * DD_NW + wave; cb < a.ncb; cb += (int64_t)gridDim.x * DD_NW) {
    int64_t r = cb;
    const int wb = (int)(r % a.wblks); r /= a.wblks;
    const int h = (int)(r % Hc); r /= Hc;
    const int d = (int)(r % Dc);
    const int n = (int)(r / Dc);
    const int wv = wb * 32 + col;
    const __amdgpu_buffer_rsrc_t rs_y = db_rsrc(dy + n * a.y.nstride, (uint32_t)a.y.nstride * 2);
    const int vbase = wv < Wc ? 2 * (half * (int)a.y.cstride + (2 * d + a.y.hlo) * (int)a.y.plane + 2 * h * Wf + 2 * wv) : DB_OOB;

    f32x16 acc[MRB];
#pragma unroll
    for (int rb = 0; rb < MRB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;

    uint32_t bqa[DD_BATCH][4], bqb[DD_BATCH][4];     // two batches of dy operands: one in flight, one being multiplied
    auto load_batch = [&](int s0, uint32_t (&dst)[DD_BATCH][4]) {
#pragma unroll
      for (int j = 0; j < DD_BATCH; ++j) {
        const int s = s0 + j;
        // the channel pair of this K-step is a scalar offset; lanes of a missing channel read nothing
        const int vo = (s < nks && 2 * s + half < a.cout) ? vbase : DB_OOB;
        const int so = __builtin_amdgcn_readfirstlane(2 * (2 * s) * (int)a.y.cstride);
#pragma unroll
        for (int ab = 0; ab < 4; ++ab)
          dst[j][ab] = __builtin_amdgcn_raw_buffer_load_b32(rs_y, vo, so + 2 * ((ab >> 1) * (int)a.y.plane + (ab & 1) * Wf), 0);
      }
    };
    auto read_a = [&](int s, uint4 (&dst)[MRB]) {
#pragma unroll
      for (int rb = 0; rb < MRB; ++rb) dst[rb] = *reinterpret_cast<const uint4*>(a_base + 16 * (2 * s * CP + rb * 32));
    };
    auto mul_batch = [&](int s0, const uint32_t (&src)[DD_BATCH][4]) {
      uint4 af[2][MRB];       // weight fragments of this K-step and of the next
      if (s0 < nks) read_a(s0, af[0]);
#pragma unroll
      for (int j = 0; j < DD_BATCH; ++j) {
        const int s = s0 + j;
        if (s < nks) {
          if (s + 1 < nks && j + 1 < DD_BATCH) read_a(s + 1, af[(j + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
          const uint4 bu = {src[j][0], src[j][1], src[j][2], src[j][3]};
          const bf16x8 B = __builtin_bit_cast(bf16x8, bu);
#pragma unroll
          for (int rb = 0; rb < MRB; ++rb)
            acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[j & 1][rb]), B, acc[rb], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    load_batch(0, bqa);
    for (int s0 = 0; s0 < nks; s0 += 2 * DD_BATCH) {
      load_batch(s0 + DD_BATCH, bqb);
      mul_batch(s0, bqa);
      load_batch(s0 + 2 * DD_BATCH, bqa);
      mul_batch(s0 + DD_BATCH, bqb);
    }

    // ---- dx[ci][d][h][wv]: accumulator register r of row block rb is channel 32 rb + 8 (r/4) + 4 half + r % 4
    // (buffer stores: the lane's voxel offset plus a scalar channel offset; a store to a channel beyond Cin or a
    //  column beyond W gets an out-of-range offset and is dropped)
    {
      const __amdgpu_buffer_rsrc_t rs_x = db_rsrc(dx + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
      const int vo = wv < Wc ? 2 * (4 * half * (int)a.x.cstride + (d + a.x.hlo) * (int)a.x.plane + h * Wc + wv) : DB_OOB;
#pragma unroll
      for (int rb = 0; rb < MRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ci_u = rb * 32 + 8 * (i / 4) + (i % 4);      // wave-uniform part of the channel
          const bool ch_ok = ci_u + 4 * half < a.cin;
          __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16(acc[rb][i]), rs_x, ch_ok ? vo : DB_OOB,
                                                __builtin_amdgcn_readfirstlane(2 * ci_u * (int)a.x.cstride), 0);
        }
    }
  }
}

template <int MRB>
h3d_status dbd_launch(void* handle, const bf16_t* dy, const bf16_t* w, bf16_t* dx, const DbdArgs& a, size_t lds_bytes,
                      hipStream_t stream) {
  static size_t attr_bytes = 0;
  if (lds_bytes > attr_bytes) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(deconv_bd_mfma_kernel<MRB>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "deconv2_bwd_data: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_bytes = lds_bytes;
  }
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  const int64_t grid = std::max<int64_t>(1, std::min<int64_t>(num_cu, cdiv(a.ncb, DD_NW)));
  hipLaunchKernelGGL((deconv_bd_mfma_kernel<MRB>), dim3((unsigned)grid), dim3(64 * DD_NW), lds_bytes, stream, dy, w, dx, a);
  return H3D_OK;
}

size_t dbd_lds_bytes(int cin, int cout) {
  const int mrb = (int)cdiv(cin, 32);
  return (size_t)((cout + 1) / 2 * 2) * ((32 * mrb) | 1) * 16;
}

}  // namespace

bool deconv_bd_mfma_supported(const h3d_tensor* dx, const h3d_tensor* dy, const void* w) {
  if (dx->dtype != H3D_BF16 || dx->c < 1 || dx->c > 128 || dy->c < 1) return false;
  if ((uintptr_t)dy->data % 4 != 0 || (uintptr_t)w % 16 != 0) return false;
  if (dbd_lds_bytes(dx->c, dy->c) > 160 * 1024) return false;
  const int64_t ys = (int64_t)dy->c * (dy->halo_lo + dy->d + dy->halo_hi) * dy->h * dy->w * 2;
  const int64_t xs = (int64_t)dx->c * (dx->halo_lo + dx->d + dx->halo_hi) * dx->h * dx->w * 2;
  return ys < ((int64_t)1 << 31) && xs < ((int64_t)1 << 31);
}

h3d_status deconv_bd_mfma(void* handle, const h3d_tensor* dy, const void* w, h3d_tensor* dx, hipStream_t stream) {
  DbdArgs a;
  a.x = make_geo(dx); a.y = make_geo(dy);
  a.cin = dx->c; a.cout = dy->c;
  a.wblks = (int)cdiv(dx->w, 32);
  a.ncb = (int64_t)dx->n * dx->d * dx->h * a.wblks;
  if (a.ncb == 0) return H3D_OK;
  const size_t lds_bytes = dbd_lds_bytes(a.cin, a.cout);
  const int mrb = (int)cdiv(a.cin, 32);
  const bf16_t* yp = (const bf16_t*)dy->data;
  const bf16_t* wp = (const bf16_t*)w;
  bf16_t* xp = (bf16_t*)dx->data;
  h3d_status st;
  if (mrb == 4) st = dbd_launch<4>(handle, yp, wp, xp, a, lds_bytes, stream);
  else if (mrb == 3) st = dbd_launch<3>(handle, yp, wp, xp, a, lds_bytes, stream);
  else if (mrb == 2) st = dbd_launch<2>(handle, yp, wp, xp, a, lds_bytes, stream);
  else st = dbd_launch<1>(handle, yp, wp, xp, a, lds_bytes, stream);
  if (st != H3D_OK) return st;
  return launch_status(handle, "deconv2_bwd_data_mfma");
}

}  // namespace h3d

// ---------------------------------------------------------------------------------------------------
// Forward of the transposed convolution:
//
//   y[co][2d+a][2h+b][2w+c] = bias[co] + sum over ci of W[ci][co][a,b,c] * x[ci][d,h,w]
//
// a GEMM with rows (co, k = (a,b,c)), columns = coarse voxels and the contraction over ci.  NCDHW keeps
// channels a whole volume apart, so (as in the 3x3x3 kernels) the x tile is transposed on its way into
// LDS: 16-byte units of 8 channels, [ci-group][voxel].  Eight wavefronts share the staged tile; wavefront
// w owns the row blocks w, w+8, ... and keeps their weight fragments (pre-packed in fragment order) in
// registers for the whole persistent workgroup.  In an accumulator the two parities c of a (co,a,b) are
// adjacent registers of one lane, so every lane stores whole dwords and consecutive lanes write
// consecutive dwords of a fine row.
namespace h3d {
namespace {

constexpr int DF_NW = 8;
constexpr int DF_CBI = 8;        // 32-voxel column blocks staged per iteration (one per wavefront)

struct DfwArgs {
  Geo x, y;
  int cin, cout;
  int wblks;
  int64_t ncb;
};

// wp: [row block][K-step][lane][8] bf16; lane l, element e: row 32 rb + l % 32 = 8 co + k, channel 16 ks + 8 (l/32) + e
__global__ void deconv_fw_pack_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int cin, int cout, int nrb, int ks) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)nrb * ks * 512) return;
  const int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  int64_t r = i >> 9;
  const int s = (int)(r % ks), rb = (int)(r / ks);
  const int row = rb * 32 + (lane & 31), co = row >> 3, k = row & 7, ci = s * 16 + (lane >> 5) * 8 + e;
  wp[i] = (co < cout && ci < cin) ? w[((int64_t)ci * cout + co) * 8 + k] : (bf16_t)0;
}

template <int RBW, int KS>
__global__ void __launch_bounds__(64 * DF_NW, 2) deconv_fw_mfma_kernel(const bf16_t* __restrict__ x, const uint4* __restrict__ wp,
                                                                     const float* __restrict__ bias, bf16_t* __restrict__ y,
                                                                     DfwArgs a) {
  constexpr int NCIG = 2 * KS;                     // groups of 8 input channels
  constexpr int CBU = NCIG * 32 + 4;               // LDS units of one column block: [ci-group][32 voxels] (+4: staggers the blocks)
  extern __shared__ uint4 lds[];                   // [2 buffers][DF_CBI][CBU]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int Wc = a.x.w, Hc = a.x.h, Dc = a.x.d, Wf = a.y.w;
  const int nrb = (8 * a.cout + 31) / 32;

  // ---- this wavefront's weight fragments
  uint4 A[RBW][KS];
#pragma unroll
  for (int j = 0; j < RBW; ++j) {
    const int rb = wave + DF_NW * j;
#pragma unroll
    for (int s = 0; s < KS; ++s) A[j][s] = rb < nrb ? wp[((int64_t)rb * KS + s) * 64 + lane] : uint4{0, 0, 0, 0};
  }

  float bv[RBW][4];
#pragma unroll
  for (int j = 0; j < RBW; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int co = 4 * (wave + DF_NW * j) + q;
      bv[j][q] = (bias && co < a.cout) ? bias[co] : 0.f;
    }

  const int ncb = (int)a.ncb;
  const int it0 = blockIdx.x * DF_CBI, it_stride = gridDim.x * DF_CBI;
  auto decode = [&](int cb, int& n, int& d, int& h, int& w0) {
    int r = cb;
    w0 = (r % a.wblks) * 32; r /= a.wblks;
    h = r % Hc; r /= Hc;
    d = r % Dc;
    n = r / Dc;
  };
  // staging: a lane takes one (ci-group, group of 8 voxels) item of its wavefront's column block per round
  constexpr int SROUNDS = (NCIG * 4 + 63) / 64;
  u32x4 sv[SROUNDS][8];
  auto stage_load = [&](int cb0) {
    const int cb = cb0 + wave;
    int n, d, h, w0;
    decode(cb < ncb ? cb : 0, n, d, h, w0);
    const __amdgpu_buffer_rsrc_t rs = db_rsrc(x + n * a.x.nstride, (uint32_t)a.x.nstride * 2);
#pragma unroll
    for (int r = 0; r < SROUNDS; ++r) {
      const int item = lane + 64 * r, cig = item >> 2, vg = item & 3;
      const int wv = w0 + 8 * vg;
      const bool ok = cb < ncb && cig < NCIG && wv + 8 <= Wc;
      const int base = 2 * (cig * 8 * (int)a.x.cstride + (d + a.x.hlo) * (int)a.x.plane + h * Wc + wv);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        sv[r][e] = __builtin_amdgcn_raw_buffer_load_b128(rs, (ok && cig * 8 + e < a.cin) ? base : DB_OOB,
                                                         __builtin_amdgcn_readfirstlane(2 * e * (int)a.x.cstride), 0);
    }
  };
  auto stage_store = [&](int buf) {
    uint4* dst0 = lds + (buf * DF_CBI + wave) * CBU;
#pragma unroll
    for (int r = 0; r < SROUNDS; ++r) {
      const int item = lane + 64 * r, cig = item >> 2, vg = item & 3;
      if (cig >= NCIG) continue;
      uint4* dst = dst0 + cig * 32 + 8 * vg;
#pragma unroll
      for (int j = 0; j < 4; ++j) {       // dword j of each channel = voxels 2j, 2j+1 of the group
        uint4 u0, u1;
        u0.x = __builtin_amdgcn_perm(sv[r][1][j], sv[r][0][j], 0x05040100); u1.x = __builtin_amdgcn_perm(sv[r][1][j], sv[r][0][j], 0x07060302);
        u0.y = __builtin_amdgcn_perm(sv[r][3][j], sv[r][2][j], 0x05040100); u1.y = __builtin_amdgcn_perm(sv[r][3][j], sv[r][2][j], 0x07060302);
        u0.z = __builtin_amdgcn_perm(sv[r][5][j], sv[r][4][j], 0x05040100); u1.z = __builtin_amdgcn_perm(sv[r][5][j], sv[r][4][j], 0x07060302);
        u0.w = __builtin_amdgcn_perm(sv[r][7][j], sv[r][6][j], 0x05040100); u1.w = __builtin_amdgcn_perm(sv[r][7][j], sv[r][6][j], 0x07060302);
        dst[2 * j] = u0;
        dst[2 * j + 1] = u1;
      }
    }
  };

  if (it0 < ncb) { stage_load(it0); stage_store(0); }
  __syncthreads();
  int buf = 0;
  for (int cb0 = it0; cb0 < ncb; cb0 += it_stride, buf ^= 1) {
    const bool more = cb0 + it_stride < ncb;
    if (more) stage_load(cb0 + it_stride);       // in flight during this iteration's MFMAs
#pragma unroll 1
    for (int c = 0; c < DF_CBI; ++c) {
      const int cb = cb0 + c;
      if (cb >= ncb) break;
      int n, d, h, w0;
      decode(cb, n, d, h, w0);
      const uint4* bp = lds + (buf * DF_CBI + c) * CBU + half * 32 + col;
      f32x16 acc[RBW];
#pragma unroll
      for (int j = 0; j < RBW; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bf16x8 B = __builtin_bit_cast(bf16x8, bp[s * 64]);
#pragma unroll
        for (int j = 0; j < RBW; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[j][s]), B, acc[j], 0, 0, 0);
      }
      // ---- rows 32 rb + 8 (i/4) + 4 half + i % 4 = 8 co + k: co = 4 rb + i / 4, a = half, b = (i % 4) / 2, c = i % 2
      const __amdgpu_buffer_rsrc_t rs_y = db_rsrc(y + n * a.y.nstride, (uint32_t)a.y.nstride * 2);
      const int wv = w0 + col;
      const int vo = wv < Wc ? 2 * ((2 * d + half + a.y.hlo) * (int)a.y.plane + 2 * h * Wf + 2 * wv) : DB_OOB;
#pragma unroll
      for (int j = 0; j < RBW; ++j) {
        const int rb = wave + DF_NW * j;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int co = 4 * rb + q;
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const uint32_t pk = pack_bf16x2(acc[j][4 * q + 2 * b] + bv[j][q], acc[j][4 * q + 2 * b + 1] + bv[j][q]);
            __builtin_amdgcn_raw_buffer_store_b32(pk, rs_y, co < a.cout ? vo : DB_OOB,
                                                  __builtin_amdgcn_readfirstlane(2 * (co * (int)a.y.cstride + b * Wf)), 0);
          }
        }
      }
    }
    if (more) stage_store(buf ^ 1);
    __syncthreads();
  }
}

template <int RBW, int KS>
h3d_status dfw_launch(void* handle, const bf16_t* x, const uint4* wp, const float* bias, bf16_t* y, const DfwArgs& a,
                      hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)2 * DF_CBI * (2 * KS * 32 + 4) * 16;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(deconv_fw_mfma_kernel<RBW, KS>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return fail(handle, H3D_EHIP, "deconv2_fwd: cannot set the dynamic LDS size to %zu bytes", lds_bytes);
    attr_set = true;
  }
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  const int64_t grid = std::max<int64_t>(1, std::min<int64_t>(num_cu, cdiv(a.ncb, DF_CBI)));
  hipLaunchKernelGGL((deconv_fw_mfma_kernel<RBW, KS>), dim3((unsigned)grid), dim3(64 * DF_NW), lds_bytes, stream, x, wp, bias, y, a);
  return H3D_OK;
}

}  // namespace

bool deconv_fw_mfma_supported(const h3d_tensor* x, const h3d_tensor* y) {
  if (x->dtype != H3D_BF16 || x->c < 1 || x->c > 128 || y->c < 1 || y->c > 64 || x->w % 8 != 0) return false;
  if ((uintptr_t)x->data % 16 != 0 || (uintptr_t)y->data % 4 != 0) return false;
  const int64_t xs = (int64_t)x->c * (x->halo_lo + x->d + x->halo_hi) * x->h * x->w * 2;
  const int64_t ys = (int64_t)y->c * (y->halo_lo + y->d + y->halo_hi) * y->h * y->w * 2;
  const int64_t ncb = (int64_t)x->n * x->d * x->h * cdiv(x->w, 32);
  return xs < ((int64_t)1 << 31) && ys < ((int64_t)1 << 31) && ncb < ((int64_t)1 << 30);
}

size_t deconv_fw_mfma_ws_bytes(const h3d_tensor* x, const h3d_tensor* y) {
  const int ks = x->c > 64 ? 8 : 4, nrb = (int)cdiv(8 * (int64_t)y->c, 32);
  return (size_t)nrb * ks * 1024;
}

h3d_status deconv_fw_mfma(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y, void* ws,
                          size_t ws_bytes, hipStream_t stream) {
  DfwArgs a;
  a.x = make_geo(x); a.y = make_geo(y);
  a.cin = x->c; a.cout = y->c;
  a.wblks = (int)cdiv(x->w, 32);
  a.ncb = (int64_t)x->n * x->d * x->h * a.wblks;
  if (a.ncb == 0) return H3D_OK;
  if (!ws || ws_bytes < deconv_fw_mfma_ws_bytes(x, y) || (uintptr_t)ws % 16) return fail(handle, H3D_EWORKSPACE, "deconv2_fwd: workspace too small or misaligned");
  const int ks = a.cin > 64 ? 8 : 4, nrb = (int)cdiv(8 * (int64_t)a.cout, 32), rbw = (int)cdiv(nrb, DF_NW);
  hipLaunchKernelGGL(deconv_fw_pack_kernel, dim3((unsigned)cdiv((int64_t)nrb * ks * 512, 256)), dim3(256), 0, stream, (const bf16_t*)w,
                     (bf16_t*)ws, a.cin, a.cout, nrb, ks);
  const bf16_t* xp = (const bf16_t*)x->data;
  bf16_t* yp = (bf16_t*)y->data;
  const uint4* wq = (const uint4*)ws;
  h3d_status st;
  if (ks == 8) st = rbw == 2 ? dfw_launch<2, 8>(handle, xp, wq, bias, yp, a, stream) : dfw_launch<1, 8>(handle, xp, wq, bias, yp, a, stream);
  else st = rbw == 2 ? dfw_launch<2, 4>(handle, xp, wq, bias, yp, a, stream) : dfw_launch<1, 4>(handle, xp, wq, bias, yp, a, stream);
  if (st != H3D_OK) return st;
  return launch_status(handle, "deconv2_fwd_mfma");
}

}  // namespace h3d
