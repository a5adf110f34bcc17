// Bit-exact strided-run copies: halo pack / unpack / zero-fill of the depth faces and channel
// concat / split.  A depth face of an N,C,D,H,W slab is n*c contiguous runs of width*h*w elements,
// so all of these are one kernel: copy `nruns` runs of `run_bytes` bytes, run r = (i, j) with
// i = r / inner, j = r % inner, at src + i*src_outer + j*src_inner (bytes), same for dst.
// HBM-bound; 16-byte accesses whenever every address involved is 16-byte aligned.
#include "common.h"

namespace h3d {

struct RunCopy {
  const char* src;  // nullptr: write zeros
  char* dst;
  int64_t nruns, inner;
  int64_t src_outer, src_inner, dst_outer, dst_inner;
  int64_t run_bytes;
  int64_t chunks_per_run;  // chunk = 256 threads * UNROLL * sizeof(V)
};

template <typename V, int UNROLL>
__global__ void __launch_bounds__(256) copy_runs_kernel(RunCopy a) {
  const int64_t blk = blockIdx.x;
  const int64_t r = blk / a.chunks_per_run, ch = blk % a.chunks_per_run;
  if (r >= a.nruns) return;
  const int64_t i = r / a.inner, j = r % a.inner;
  const int64_t nvec = a.run_bytes / (int64_t)sizeof(V);
  V* d = reinterpret_cast<V*>(a.dst + i * a.dst_outer + j * a.dst_inner);
  const V* s = a.src ? reinterpret_cast<const V*>(a.src + i * a.src_outer + j * a.src_inner) : nullptr;
  const int64_t base = ch * (256 * UNROLL) + threadIdx.x;
  V v[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    int64_t e = base + u * 256;
    if (s) {
      if (e < nvec) v[u] = s[e];
    } else {
      memset(&v[u], 0, sizeof(V));
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    int64_t e = base + u * 256;
    if (e < nvec) d[e] = v[u];
  }
}

static h3d_status copy_runs(void* handle, RunCopy a, hipStream_t stream, const char* what) {
  if (a.nruns <= 0 || a.run_bytes <= 0) return H3D_OK;
  auto al = [](int64_t v, int64_t m) { return (v % m) == 0; };
  uintptr_t ps = (uintptr_t)a.src, pd = (uintptr_t)a.dst;
  bool v16 = al(ps, 16) && al(pd, 16) && al(a.src_outer, 16) && al(a.src_inner, 16) && al(a.dst_outer, 16) &&
             al(a.dst_inner, 16) && al(a.run_bytes, 16);
  bool v4 = al(ps, 4) && al(pd, 4) && al(a.src_outer, 4) && al(a.src_inner, 4) && al(a.dst_outer, 4) &&
            al(a.dst_inner, 4) && al(a.run_bytes, 4);
  constexpr int U = 4;
  if (v16) {
    a.chunks_per_run = cdiv(a.run_bytes / 16, 256 * U);
    int64_t grid = a.nruns * a.chunks_per_run;
    if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "%s: too many blocks", what);
    hipLaunchKernelGGL((copy_runs_kernel<uint4, U>), dim3((unsigned)grid), dim3(256), 0, stream, a);
  } else if (v4) {
    a.chunks_per_run = cdiv(a.run_bytes / 4, 256 * U);
    int64_t grid = a.nruns * a.chunks_per_run;
    if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "%s: too many blocks", what);
    hipLaunchKernelGGL((copy_runs_kernel<uint32_t, U>), dim3((unsigned)grid), dim3(256), 0, stream, a);
  } else {
    a.chunks_per_run = cdiv(a.run_bytes / 2, 256 * U);  // every dtype here is 2 or 4 bytes wide
    int64_t grid = a.nruns * a.chunks_per_run;
    if (grid >= ((int64_t)1 << 31)) return fail(handle, H3D_EINVAL, "%s: too many blocks", what);
    hipLaunchKernelGGL((copy_runs_kernel<uint16_t, U>), dim3((unsigned)grid), dim3(256), 0, stream, a);
  }
  return launch_status(handle, what);
}

// Copy the interior of channels [c0, c0+nc) of `src` to channels [c1, c1+nc) of `dst`.
h3d_status copy_channels(void* handle, const h3d_tensor* src, int c0, h3d_tensor* dst, int c1, int nc,
                         hipStream_t stream, const char* what) {
  const int64_t es = elt_size(src->dtype);
  Geo gs = make_geo(src), gd = make_geo(dst);
  RunCopy a{};
  a.src = (const char*)src->data + (c0 * gs.cstride + (int64_t)gs.hlo * gs.plane) * es;
  a.dst = (char*)dst->data + (c1 * gd.cstride + (int64_t)gd.hlo * gd.plane) * es;
  a.nruns = (int64_t)src->n * nc;
  a.inner = nc;
  a.src_outer = gs.nstride * es; a.src_inner = gs.cstride * es;
  a.dst_outer = gd.nstride * es; a.dst_inner = gd.cstride * es;
  a.run_bytes = (int64_t)src->d * gs.plane * es;
  return copy_runs(handle, a, stream, what);
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_halo_bytes(const h3d_tensor* t, int width) {
  if (!t || width <= 0) return 0;
  return (size_t)t->n * t->c * width * t->h * t->w * elt_size(t->dtype);
}

static h3d_status face_args(void* handle, const h3d_tensor* t, int face, int width, bool pack, RunCopy* a) {
  H3D_TRY(check_tensor_packed(handle, t, "t"));
  if (face != H3D_FACE_D_LO && face != H3D_FACE_D_HI && face != H3D_FACE_D_BOTH) return fail(handle, H3D_EINVAL, "halo: bad face %d", face);
  if (width <= 0) return fail(handle, H3D_EINVAL, "halo: width must be positive");
  const bool both = face == H3D_FACE_D_BOTH;
  int64_t first, first_hi;  // first stored plane of the face region (of the LO region and of the HI region for D_BOTH)
  if (pack) {
    if (width > t->d) return fail(handle, H3D_EINVAL, "halo_pack: width %d exceeds interior depth %d", width, t->d);
    first_hi = t->halo_lo + t->d - width;
    first = face == H3D_FACE_D_HI ? first_hi : t->halo_lo;
  } else {
    int have = both ? (t->halo_lo < t->halo_hi ? t->halo_lo : t->halo_hi) : (face == H3D_FACE_D_LO ? t->halo_lo : t->halo_hi);
    if (width > have) return fail(handle, H3D_EHALO, "halo_unpack: width %d exceeds stored halo %d", width, have);
    first_hi = t->halo_lo + t->d;
    first = face == H3D_FACE_D_HI ? first_hi : t->halo_lo - width;
  }
  Geo g = make_geo(t);
  const int64_t es = elt_size(t->dtype);
  const int64_t nc = (int64_t)t->n * t->c;
  a->nruns = both ? 2 * nc : nc;
  a->inner = nc;            // run r = (face i = r / inner, (n, c) j = r % inner); one face: i = 0
  a->run_bytes = (int64_t)width * g.plane * es;
  // slab side: the HI region starts (first_hi - first) planes above the LO region; buffer side: the HI face follows the LO face
  const int64_t slab_off = first * g.plane * es, slab_stride = g.cstride * es;
  const int64_t slab_outer = both ? (first_hi - first) * g.plane * es : 0, buf_outer = both ? nc * a->run_bytes : 0;
  if (pack) {
    a->src = (const char*)t->data + slab_off; a->src_outer = slab_outer; a->src_inner = slab_stride;
    a->dst_outer = buf_outer; a->dst_inner = a->run_bytes;
  } else {
    a->dst = (char*)t->data + slab_off; a->dst_outer = slab_outer; a->dst_inner = slab_stride;
    a->src_outer = buf_outer; a->src_inner = a->run_bytes;
  }
  return H3D_OK;
}

extern "C" h3d_status h3d_halo_pack(void* handle, const h3d_tensor* t, int face, int width, void* buf, void* stream) {
  if (!handle) return H3D_EINVAL;
  RunCopy a{};
  H3D_TRY(face_args(handle, t, face, width, true, &a));
  if (!buf && a.nruns * a.run_bytes > 0) return fail(handle, H3D_EINVAL, "halo_pack: NULL buffer");
  a.dst = (char*)buf;
  return copy_runs(handle, a, (hipStream_t)stream, "halo_pack");
}

extern "C" h3d_status h3d_halo_unpack(void* handle, const void* buf, h3d_tensor* t, int face, int width, void* stream) {
  if (!handle) return H3D_EINVAL;
  RunCopy a{};
  H3D_TRY(face_args(handle, t, face, width, false, &a));
  a.src = (const char*)buf;  // nullptr => zero fill
  if (!buf) { a.src_inner = 0; a.src_outer = 0; }
  return copy_runs(handle, a, (hipStream_t)stream, "halo_unpack");
}

static h3d_status cat_check(void* handle, const h3d_tensor* a, const h3d_tensor* b, const h3d_tensor* o) {
  H3D_TRY(check_tensor_packed(handle, a, "a"));
  H3D_TRY(check_tensor_packed(handle, b, "b"));
  H3D_TRY(check_tensor_packed(handle, o, "out"));
  if (!same_shard(a, b) || !same_shard(a, o) || o->c != a->c + b->c)
    return fail(handle, H3D_EINVAL, "concat/split: shapes do not match (need same n,d,h,w,offsets,dtype and c = ca+cb)");
  return H3D_OK;
}

extern "C" h3d_status h3d_concat_c(void* handle, const h3d_tensor* a, const h3d_tensor* b, h3d_tensor* out, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(cat_check(handle, a, b, out));
  H3D_TRY(copy_channels(handle, a, 0, out, 0, a->c, (hipStream_t)stream, "concat_c"));
  return copy_channels(handle, b, 0, out, a->c, b->c, (hipStream_t)stream, "concat_c");
}

extern "C" h3d_status h3d_split_c(void* handle, const h3d_tensor* in, h3d_tensor* a, h3d_tensor* b, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(cat_check(handle, a, b, in));
  H3D_TRY(copy_channels(handle, in, 0, a, 0, a->c, (hipStream_t)stream, "split_c"));
  return copy_channels(handle, in, a->c, b, 0, b->c, (hipStream_t)stream, "split_c");
}
