// Pack / unpack of GENERAL faces: a box of a packed 5-D tensor [n][c][D][H][W] to / from a contiguous buffer
// [n][c][bd][bh][bw].  The depth faces of the hot path are runs of whole planes (copy.hip); a partitioning in H
// or W as well (Sec. II-B: spatial partitioning in any of the three dimensions; Sec. III-A: the packing and
// unpacking kernels of the boundary exchange, for 3^3 and 5^3 filters = faces 1 or 2 voxels wide) exchanges
// strided faces: an H face is bd*... rows of bw contiguous elements, a W face is 1 or 2 elements per row.
//
// One kernel, the vector width picked per call: a thread moves VEC contiguous elements of a box row (16 bytes
// when extents, origin and pointers allow it); consecutive threads walk w, then h, d, c, n of the BOX, so the
// buffer side is always fully coalesced and the tensor side is as contiguous as the box allows.
#include <algorithm>

#include "common.h"

namespace h3d {
namespace {

struct BoxArgs {
  int64_t total;          // threads = box elements / VEC
  int c, bd, bh, bwv;     // box extents (bwv = bw / VEC)
  int64_t sn, sc, sd, sh; // tensor strides in elements
  int64_t origin;         // element offset of the box origin inside the tensor
};

template <typename V, int DIR>   // DIR 0: tensor -> buffer, 1: buffer -> tensor, 2: zero -> tensor
__global__ void __launch_bounds__(256) box_copy_kernel(const V* __restrict__ src, V* __restrict__ dst, BoxArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.total) return;
  int64_t t = i;
  const int wv = (int)(t % a.bwv); t /= a.bwv;
  const int h = (int)(t % a.bh); t /= a.bh;
  const int d = (int)(t % a.bd); t /= a.bd;
  const int c = (int)(t % a.c);
  const int64_t n = t / a.c;
  // strides and origin are multiples of the vector width, so the tensor offset is a whole number of vectors
  const int64_t toff = a.origin + n * a.sn + c * a.sc + d * a.sd + h * a.sh + wv;
  if (DIR == 0) dst[i] = src[toff];
  else if (DIR == 1) dst[toff] = src[i];
  else {
    V z;
    memset(&z, 0, sizeof(V));
    dst[toff] = z;
  }
}

template <typename V>
h3d_status box_launch(int dir, const void* src, void* dst, const BoxArgs& a, hipStream_t stream) {
  const int64_t grid = cdiv(a.total, 256);
  if (dir == 0) hipLaunchKernelGGL((box_copy_kernel<V, 0>), dim3((unsigned)grid), dim3(256), 0, stream, (const V*)src, (V*)dst, a);
  else if (dir == 1) hipLaunchKernelGGL((box_copy_kernel<V, 1>), dim3((unsigned)grid), dim3(256), 0, stream, (const V*)src, (V*)dst, a);
  else hipLaunchKernelGGL((box_copy_kernel<V, 2>), dim3((unsigned)grid), dim3(256), 0, stream, (const V*)nullptr, (V*)dst, a);
  return H3D_OK;
}

h3d_status box_copy(void* handle, int dir, const void* tensor_or_buf_src, void* dst, const void* tensor, int dtype, int n, int c, int D, int H,
                    int W, const h3d_box* b, const void* buf, hipStream_t stream, const char* what) {
  if (dtype != H3D_F32 && dtype != H3D_BF16) return fail(handle, H3D_EINVAL, "%s: bad dtype %d", what, dtype);
  if (!b || !tensor) return fail(handle, H3D_EINVAL, "%s: NULL pointer", what);
  if (n < 0 || c < 0 || D < 0 || H < 0 || W < 0) return fail(handle, H3D_EINVAL, "%s: negative extent", what);
  if (b->d0 < 0 || b->h0 < 0 || b->w0 < 0 || b->bd < 0 || b->bh < 0 || b->bw < 0 || (int64_t)b->d0 + b->bd > D ||
      (int64_t)b->h0 + b->bh > H || (int64_t)b->w0 + b->bw > W)
    return fail(handle, H3D_EINVAL, "%s: box [%d+%d, %d+%d, %d+%d] outside the tensor %dx%dx%d", what, b->d0, b->bd, b->h0, b->bh, b->w0,
                b->bw, D, H, W);
  const int64_t elems = (int64_t)n * c * b->bd * b->bh * b->bw;
  if (elems == 0) return H3D_OK;
  if (dir != 2 && !buf) return fail(handle, H3D_EINVAL, "%s: NULL buffer", what);
  const int es = (int)elt_size(dtype);
  // widest vector (bytes) that divides the row length, the origin, the row pitch and both pointers
  int vb = 16;
  auto fits = [&](int bytes) {
    const int ve = bytes / es;
    return ve >= 1 && b->bw % ve == 0 && b->w0 % ve == 0 && W % ve == 0 && (uintptr_t)tensor % bytes == 0 &&
           (dir == 2 || (uintptr_t)buf % bytes == 0);
  };
  while (vb > es && !fits(vb)) vb /= 2;
  const int ve = vb / es;
  BoxArgs a;
  a.c = c; a.bd = b->bd; a.bh = b->bh; a.bwv = b->bw / ve;
  a.total = elems / ve;
  a.sh = W / ve; a.sd = (int64_t)H * W / ve; a.sc = (int64_t)D * H * W / ve; a.sn = (int64_t)c * D * H * W / ve;
  a.origin = (((int64_t)b->d0 * H + b->h0) * W + b->w0) / ve;
  if (cdiv(a.total, 256) >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "%s: too many blocks", what);
  (void)tensor_or_buf_src;
  const void* src = dir == 0 ? tensor : buf;
  switch (vb) {
    case 16: box_launch<uint4>(dir, src, dst, a, stream); break;
    case 8: box_launch<uint2>(dir, src, dst, a, stream); break;
    case 4: box_launch<uint32_t>(dir, src, dst, a, stream); break;
    default: box_launch<uint16_t>(dir, src, dst, a, stream); break;
  }
  return launch_status(handle, what);
}

}  // namespace
}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_box_bytes(int dtype, int n, int c, const h3d_box* box) {
  if (!box || n <= 0 || c <= 0 || box->bd <= 0 || box->bh <= 0 || box->bw <= 0 || (dtype != H3D_F32 && dtype != H3D_BF16)) return 0;
  return (size_t)n * c * box->bd * box->bh * box->bw * elt_size(dtype);
}

extern "C" h3d_status h3d_box_pack(void* handle, const void* t, int dtype, int n, int c, int D, int H, int W, const h3d_box* box, void* buf,
                                   void* stream) {
  if (!handle) return H3D_EINVAL;
  return box_copy(handle, 0, t, buf, t, dtype, n, c, D, H, W, box, buf, (hipStream_t)stream, "box_pack");
}

extern "C" h3d_status h3d_box_unpack(void* handle, const void* buf, void* t, int dtype, int n, int c, int D, int H, int W, const h3d_box* box,
                                     void* stream) {
  if (!handle) return H3D_EINVAL;
  return box_copy(handle, buf ? 1 : 2, buf, t, t, dtype, n, c, D, H, W, box, buf, (hipStream_t)stream, "box_unpack");
}
