// Entry points of the 3x3x3 convolution passes: host-side validation of shapes, halos and
// workspace, then dispatch to the kernel family that fits the shape.
#include <algorithm>

#include "common.h"

namespace h3d {
// conv_direct.hip
size_t direct_fwd_ws_bytes(int cin_k, int cout_k);
size_t direct_bf_ws_bytes(const h3d_tensor* x, int cout);
template <typename T>
h3d_status conv3d_direct(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                         h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                         hipStream_t stream);
template <typename T>
h3d_status bwd_filter_direct(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                             float* db, float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream);
// conv_f32_mfma.hip
bool f32_mfma_fwd_supported(const h3d_tensor* in, const h3d_tensor* out);
size_t f32_mfma_fwd_ws_bytes(int cin_k, int cout_k);
h3d_status conv3d_f32_mfma(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                           h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                           hipStream_t stream);
bool f32_mfma_bf_supported(const h3d_tensor* x, const h3d_tensor* dz);
size_t f32_mfma_bf_ws_bytes(const h3d_tensor* x, int cout);
h3d_status bwd_filter_f32_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                               float* db, float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream);
// conv_small_cin.hip
bool c4_fwd_supported(const h3d_tensor* in, const h3d_tensor* out);
bool c4_fwd_pool_supported(const h3d_tensor* in, const h3d_tensor* z, const h3d_tensor* y);
h3d_status conv3d_fwd_c4_pool(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, h3d_tensor* y,
                              void* mask, float out_slope, void* ws, size_t ws_bytes, hipStream_t stream);
h3d_status pool_shapes_check(void* handle, const h3d_tensor* big, const h3d_tensor* small, const char* what);
bool c4_roll_supported(const h3d_tensor* in, const h3d_tensor* z);
size_t c4_roll_ws_bytes();
h3d_status conv3d_fwd_c4_roll(void* handle, const h3d_tensor* in, const void* w, const float* bias, const h3d_tensor* z, const h3d_tensor* y,
                              void* mask, float out_slope, void* ws, size_t ws_bytes, hipStream_t stream);
size_t c4_fwd_ws_bytes(const h3d_tensor* out);
h3d_status conv3d_fwd_c4(void* handle, const h3d_tensor* in, const void* w, const float* bias, h3d_tensor* out, float out_slope,
                         void* ws, size_t ws_bytes, hipStream_t stream);
// conv_mfma.hip
bool mfma_fwd_supported(const h3d_tensor* in, const h3d_tensor* out);
size_t mfma_fwd_ws_bytes(const h3d_tensor* in, const h3d_tensor* out);
h3d_status conv3d_mfma(void* handle, const h3d_tensor* in, const h3d_tensor* mask, const void* w, const float* bias,
                       h3d_tensor* out, bool transpose, float out_slope, float mask_slope, void* ws, size_t ws_bytes,
                       hipStream_t stream);
bool mfma_bf_supported(const h3d_tensor* x, const h3d_tensor* dz);
size_t mfma_bf_ws_bytes(const h3d_tensor* x, const h3d_tensor* dz);
h3d_status bwd_filter_mfma(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z, float* dw,
                           float* db, float mask_slope, void* ws, size_t ws_bytes, hipStream_t stream);

static h3d_status check_act(void* handle, int act) {
  if (act != H3D_ACT_NONE && act != H3D_ACT_RELU && act != H3D_ACT_LEAKY) return fail(handle, H3D_EINVAL, "bad activation %d", act);
  return H3D_OK;
}

// in -> out correlation geometry check shared by forward and backward-data
static h3d_status check_pair(void* handle, const h3d_tensor* in, const h3d_tensor* out, const char* what) {
  if (!same_shard(in, out)) return fail(handle, H3D_EINVAL, "%s: input and output must agree in n,d,h,w,d_offset,d_global,dtype", what);
  if (!halo_covers(in, -(int64_t)out->halo_lo, (int64_t)out->d + out->halo_hi))
    return fail(handle, H3D_EHALO, "%s: input stores halo %d/%d but output planes [-%d,%d) need a plane that is inside the volume and not stored",
                what, in->halo_lo, in->halo_hi, out->halo_lo, out->d + out->halo_hi);
  return H3D_OK;
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_conv3d_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* z) {
  if (!handle || !x || !z) return 0;
  size_t b = 0;
  switch (op) {
    case H3D_OP_FWD:       // x: input, z: output
      if (c4_fwd_supported(x, z)) b = std::max(c4_fwd_ws_bytes(z), c4_roll_ws_bytes());
      [[fallthrough]];
    case H3D_OP_BWD_DATA:  // x: dz (input of the correlation), z: dx
      b = std::max(b, direct_fwd_ws_bytes(x->c, z->c));
      if (mfma_fwd_supported(x, z)) b = std::max(b, mfma_fwd_ws_bytes(x, z));
      if (f32_mfma_fwd_supported(x, z)) b = std::max(b, f32_mfma_fwd_ws_bytes(x->c, z->c));
      break;
    case H3D_OP_BWD_FILTER:  // x: activations, z: dz
      // the size of the one kernel family h3d_conv3d_bwd_filter gives these shapes to (same order of tests as there)
      if (mfma_bf_supported(x, z)) b = mfma_bf_ws_bytes(x, z);
      else if (f32_mfma_bf_supported(x, z)) b = f32_mfma_bf_ws_bytes(x, z->c);
      else b = direct_bf_ws_bytes(x, z->c);
      break;
    default:
      return 0;
  }
  return (b + 255) & ~(size_t)255;
}

extern "C" h3d_status h3d_conv3d_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* z,
                                     int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor(handle, x, "x"));
  H3D_TRY(check_tensor(handle, z, "z"));
  H3D_TRY(check_act(handle, act));
  if (!w && x->c * z->c > 0) return fail(handle, H3D_EINVAL, "conv3d_fwd: NULL weights");
  H3D_TRY(check_pair(handle, x, z, "conv3d_fwd"));
  const float slope = act_slope(act, alpha);
  hipStream_t s = (hipStream_t)stream;
  if (c4_roll_supported(x, z)) return conv3d_fwd_c4_roll(handle, x, w, bias, z, nullptr, nullptr, slope, ws, ws_bytes, s);
  if (c4_fwd_supported(x, z)) return conv3d_fwd_c4(handle, x, w, bias, z, slope, ws, ws_bytes, s);
  if (mfma_fwd_supported(x, z)) return conv3d_mfma(handle, x, nullptr, w, bias, z, false, slope, 1.f, ws, ws_bytes, s);
  if (f32_mfma_fwd_supported(x, z)) return conv3d_f32_mfma(handle, x, nullptr, w, bias, z, false, slope, 1.f, ws, ws_bytes, s);
  if (x->dtype == H3D_F32) return conv3d_direct<float>(handle, x, nullptr, w, bias, z, false, slope, 1.f, ws, ws_bytes, s);
  return conv3d_direct<bf16_t>(handle, x, nullptr, w, bias, z, false, slope, 1.f, ws, ws_bytes, s);
}

extern "C" h3d_status h3d_conv3d_fwd_pool(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* z,
                                          h3d_tensor* y, void* mask, int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!z || !y) return fail(handle, H3D_EINVAL, "conv3d_fwd_pool: NULL descriptor");
  h3d_tensor zc = *z;                    // z may be shape-only (data == NULL: the unpooled output is not stored)
  if (!zc.data) zc.data = y->data;
  H3D_TRY(check_tensor(handle, x, "x"));
  H3D_TRY(check_tensor(handle, &zc, "z"));
  H3D_TRY(check_tensor_packed(handle, y, "y"));
  H3D_TRY(check_act(handle, act));
  if (!w && x->c * z->c > 0) return fail(handle, H3D_EINVAL, "conv3d_fwd_pool: NULL weights");
  H3D_TRY(check_pair(handle, x, &zc, "conv3d_fwd_pool"));
  H3D_TRY(pool_shapes_check(handle, &zc, y, "conv3d_fwd_pool"));
  // what the mask pass of the three-pass route would refuse is refused here, before anything is enqueued
  if (mask && z->w % 8) return fail(handle, H3D_EUNSUPPORTED, "conv3d_fwd_pool: a mask needs w to be a multiple of 8");
  if (!is_packed(z)) return fail(handle, H3D_EUNSUPPORTED, "conv3d_fwd_pool: z must be a packed tensor (the pooling pass takes no plane-run views)");
  const float slope = act_slope(act, alpha);
  hipStream_t s = (hipStream_t)stream;
  if (c4_fwd_pool_supported(x, z, y) && c4_roll_supported(x, z))
    return conv3d_fwd_c4_roll(handle, x, w, bias, z, y, mask, slope, ws, ws_bytes, s);
  if (c4_fwd_pool_supported(x, z, y)) return conv3d_fwd_c4_pool(handle, x, w, bias, z, y, mask, slope, ws, ws_bytes, s);
  // other shapes: the three passes one after the other (the unpooled output must then be stored)
  if (!z->data) return fail(handle, H3D_EUNSUPPORTED, "conv3d_fwd_pool: this shape has no fused kernel, z must be stored");
  H3D_TRY(h3d_conv3d_fwd(handle, x, w, bias, z, act, alpha, ws, ws_bytes, stream));
  H3D_TRY(h3d_pool3d_fwd(handle, z, y, H3D_POOL_AVG, stream));
  if (mask) H3D_TRY(h3d_act_mask(handle, z, mask, stream));
  return H3D_OK;
}

extern "C" h3d_status h3d_conv3d_bwd_data(void* handle, const h3d_tensor* dz, const h3d_tensor* z, const void* w,
                                          h3d_tensor* dx, int act, float alpha, void* ws, size_t ws_bytes, void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor(handle, dz, "dz"));
  H3D_TRY(check_tensor(handle, dx, "dx"));
  H3D_TRY(check_act(handle, act));
  if (!w && dz->c * dx->c > 0) return fail(handle, H3D_EINVAL, "conv3d_bwd_data: NULL weights");
  H3D_TRY(check_pair(handle, dz, dx, "conv3d_bwd_data"));
  if (act == H3D_ACT_NONE) z = nullptr;
  if (z) {
    H3D_TRY(check_tensor(handle, z, "z"));
    if (!same_shard(z, dz) || z->c != dz->c) return fail(handle, H3D_EINVAL, "conv3d_bwd_data: z and dz shapes differ");
    if (!halo_covers(z, -(int64_t)dx->halo_lo, (int64_t)dx->d + dx->halo_hi))
      return fail(handle, H3D_EHALO, "conv3d_bwd_data: z does not store the planes dz is read at");
  }
  const float slope = act_slope(act, alpha);
  hipStream_t s = (hipStream_t)stream;
  if (mfma_fwd_supported(dz, dx)) return conv3d_mfma(handle, dz, z, w, nullptr, dx, true, 1.f, slope, ws, ws_bytes, s);
  if (f32_mfma_fwd_supported(dz, dx)) return conv3d_f32_mfma(handle, dz, z, w, nullptr, dx, true, 1.f, slope, ws, ws_bytes, s);
  if (dz->dtype == H3D_F32) return conv3d_direct<float>(handle, dz, z, w, nullptr, dx, true, 1.f, slope, ws, ws_bytes, s);
  return conv3d_direct<bf16_t>(handle, dz, z, w, nullptr, dx, true, 1.f, slope, ws, ws_bytes, s);
}

extern "C" h3d_status h3d_conv3d_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z,
                                            float* dw, float* db, int act, float alpha, void* ws, size_t ws_bytes,
                                            void* stream) {
  if (!handle) return H3D_EINVAL;
  H3D_TRY(check_tensor(handle, x, "x"));
  H3D_TRY(check_tensor(handle, dz, "dz"));
  H3D_TRY(check_act(handle, act));
  if (!same_shard(x, dz)) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: x and dz must agree in n,d,h,w,d_offset,d_global,dtype");
  if (!dw && x->c * dz->c > 0) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: NULL dw");
  if (!halo_covers(x, 0, x->d)) return fail(handle, H3D_EHALO, "conv3d_bwd_filter: x must store one halo plane on every side that is inside the volume");
  if (act == H3D_ACT_NONE) z = nullptr;
  if (z) {
    H3D_TRY(check_tensor(handle, z, "z"));
    if (!same_shard(z, dz) || z->c != dz->c) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter: z and dz shapes differ");
  }
  const float slope = act_slope(act, alpha);
  hipStream_t s = (hipStream_t)stream;
  if (mfma_bf_supported(x, dz)) return bwd_filter_mfma(handle, x, dz, z, dw, db, slope, ws, ws_bytes, s);
  if (f32_mfma_bf_supported(x, dz)) return bwd_filter_f32_mfma(handle, x, dz, z, dw, db, slope, ws, ws_bytes, s);
  if (x->dtype == H3D_F32) return bwd_filter_direct<float>(handle, x, dz, z, dw, db, slope, ws, ws_bytes, s);
  return bwd_filter_direct<bf16_t>(handle, x, dz, z, dw, db, slope, ws, ws_bytes, s);
}
