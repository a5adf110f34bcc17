// Internal definitions shared by the HIP translation units of libh3d (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "h3d.h"

namespace h3d {

h3d_status fail(void* handle, h3d_status st, const char* fmt, ...);

struct Handle {
  int device = 0;
  int num_cu = 256;
  void* scratch = nullptr;    // this device's copy of the library-owned scratch array (static_scratch.hip)
  char err[512] = {0};
  char kernel[160] = {0};     // principal kernel of the last compute call (h3d_last_kernel)
  bool kernel_noted = false;
};

// size of the library-owned scratch array behind h3d_conv3d_bwd_filter_static
#define H3D_STATIC_SCRATCH_BYTES (96u << 20)
h3d_status static_scratch_init(Handle* hd);

// Slab geometry as the kernels see it (element strides, not bytes).
struct Geo {
  int n, c, d, h, w, hlo, hhi;
  int ds;            // stored planes = hlo + d + hhi
  int64_t doff, dglob;
  int64_t plane;     // h*w
  int64_t cstride;   // ds*h*w
  int64_t nstride;   // c*ds*h*w
};

inline Geo make_geo(const h3d_tensor* t) {
  Geo g;
  g.n = t->n; g.c = t->c; g.d = t->d; g.h = t->h; g.w = t->w; g.hlo = t->halo_lo; g.hhi = t->halo_hi;
  g.ds = t->halo_lo + t->d + t->halo_hi;
  g.doff = t->d_offset; g.dglob = t->d_global;
  g.plane = (int64_t)t->h * t->w;
  g.cstride = t->c_stride ? t->c_stride : g.plane * g.ds;
  g.nstride = t->n_stride ? t->n_stride : g.cstride * t->c;
  return g;
}

inline bool is_packed(const h3d_tensor* t) { return t->c_stride == 0 && t->n_stride == 0; }
// elements spanned by one sample (all channels), with the tensor's real strides
inline int64_t sample_span(const h3d_tensor* t) {
  const int64_t cs = t->c_stride ? t->c_stride : (int64_t)(t->halo_lo + t->d + t->halo_hi) * t->h * t->w;
  return t->n_stride ? t->n_stride : cs * t->c;
}

inline size_t elt_size(int dtype) { return dtype == H3D_F32 ? 4 : 2; }

h3d_status fail(void* handle, h3d_status st, const char* fmt, ...);
h3d_status check_tensor(void* handle, const h3d_tensor* t, const char* name);          // strided plane runs allowed
h3d_status check_tensor_packed(void* handle, const h3d_tensor* t, const char* name);   // packed tensors only
// every needed in-volume input plane for output planes [lo,hi) (local indices) must be stored
bool halo_covers(const h3d_tensor* in, int64_t lo, int64_t hi);
bool same_shard(const h3d_tensor* a, const h3d_tensor* b);
h3d_status launch_status(void* handle, const char* what);   // also records `what` as the call's kernel unless one was noted
// name of the kernel that does the arithmetic of the call under way (shown by h3d_last_kernel)
void note_kernel(void* handle, const char* fmt, ...);

inline float act_slope(int act, float alpha) { return act == H3D_ACT_LEAKY ? alpha : (act == H3D_ACT_RELU ? 0.f : 1.f); }

// ---- bf16 storage helpers (device) -------------------------------------------------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two floats -> packed bf16x2 (low half = first), round to nearest even: one v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ---- global -> LDS copies without registers (buffer_load ... lds) ---------------------------------------------------
// The instruction is issued from inline assembly on purpose: the compiler's wait-count pass treats a copy into LDS as
// aliasing every later LDS read and puts "s_waitcnt vmcnt(0)" in front of the first one, which serialises a prefetch
// with the arithmetic it was meant to hide behind.  Issued this way the copies are invisible to that pass; the kernel
// itself waits (s_waitcnt vmcnt) and synchronises (barrier) before anyone reads the destination.  Hidden operations can
// only make the compiler's own vmcnt waits longer, never shorter: the counter is decremented in issue order.
typedef int h3d_i32x4 __attribute__((ext_vector_type(4)));
// raw buffer resource: byte range [base, base + bytes), accesses beyond it return zeros
__device__ __forceinline__ h3d_i32x4 lds_dma_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  h3d_i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(p >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}
// LDS byte address of a pointer into shared memory (wave-uniform)
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p);
}
// 64 lanes x 16 bytes from per-lane byte offsets `voff` of the buffer into 1 KB of LDS at `lds_byte_addr` (lane l at + 16 l)
__device__ __forceinline__ void lds_dma16(h3d_i32x4 rs, uint32_t lds_byte_addr, int voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_byte_addr), "v"(voff), "s"(rs) : "memory", "m0");
}

template <typename T> struct dtype_of;
template <> struct dtype_of<float> { static constexpr int value = H3D_F32; };
template <> struct dtype_of<bf16_t> { static constexpr int value = H3D_BF16; };

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace h3d

#define H3D_TRY(expr)                       \
  do {                                      \
    h3d_status _s = (expr);                 \
    if (_s != H3D_OK) return _s;            \
  } while (0)
