// bf16 MFMA implicit-GEMM convolution kernels (placeholder until the matrix-core path lands:
// every shape currently takes the direct kernels).
#include "common.h"

namespace h3d {
bool mfma_fwd_supported(const h3d_tensor*, const h3d_tensor*) { return false; }
size_t mfma_fwd_ws_bytes(const h3d_tensor*, const h3d_tensor*) { return 0; }
h3d_status conv3d_mfma(void* handle, const h3d_tensor*, const h3d_tensor*, const void*, const float*, h3d_tensor*, bool, float,
                       float, void*, size_t, hipStream_t) {
  return fail(handle, H3D_EUNSUPPORTED, "conv3d_mfma: not built");
}
bool mfma_bf_supported(const h3d_tensor*, const h3d_tensor*) { return false; }
size_t mfma_bf_ws_bytes(const h3d_tensor*, const h3d_tensor*) { return 0; }
h3d_status bwd_filter_mfma(void* handle, const h3d_tensor*, const h3d_tensor*, const h3d_tensor*, float*, float*, float, void*,
                           size_t, hipStream_t) {
  return fail(handle, H3D_EUNSUPPORTED, "bwd_filter_mfma: not built");
}
}  // namespace h3d
