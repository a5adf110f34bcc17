// Backward-filter for callers that cannot allocate device memory or hand over a workspace: the per-chunk partial sums
// of the split-spatial reduction live in a fixed device array owned by the library.
#include "common.h"

namespace h3d {

// One copy per GPU the library runs on, held until the process ends.  In host code the array's NAME is only a
// stand-in for the symbol; the device address is looked up once per device (h3d_create) and that pointer is what
// every launch receives.
static __device__ __align__(256) unsigned char scratch[H3D_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Called by h3d_create with the handle's device current.
h3d_status static_scratch_init(Handle* hd) {
  if (hd->device < 0 || hd->device >= kMaxDevices) return fail(hd, H3D_EINVAL, "device index %d out of range", hd->device);
  if (!g_scratch_ptr[hd->device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(hd, H3D_EHIP, "static scratch: hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[hd->device] = p;
  }
  hd->scratch = g_scratch_ptr[hd->device];
  return H3D_OK;
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_static_scratch_bytes(void) { return (size_t)H3D_STATIC_SCRATCH_BYTES; }

extern "C" h3d_status h3d_conv3d_bwd_filter_static(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z,
                                                   float* dw, float* db, int act, float alpha, void* stream) {
  if (!handle) return H3D_EINVAL;
  Handle* hd = static_cast<Handle*>(handle);
  if (!x || !dz) return fail(handle, H3D_EINVAL, "conv3d_bwd_filter_static: NULL descriptor");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != hd->device)
    return fail(handle, H3D_EINVAL, "conv3d_bwd_filter_static: the handle belongs to device %d, the current device is %d", hd->device, dev);
  if (!hd->scratch) return fail(handle, H3D_EHIP, "conv3d_bwd_filter_static: the static scratch buffer was not set up");
  const size_t need = h3d_conv3d_workspace_bytes(handle, H3D_OP_BWD_FILTER, x, dz);
  if (need > (size_t)H3D_STATIC_SCRATCH_BYTES)
    return fail(handle, H3D_EWORKSPACE, "conv3d_bwd_filter_static: these shapes need %zu bytes of scratch, the static buffer holds %zu; "
                "use h3d_conv3d_bwd_filter with a workspace", need, (size_t)H3D_STATIC_SCRATCH_BYTES);
  // every partial sum the second stage reads is written by the first stage of the same call: nothing has to start at zero
  return h3d_conv3d_bwd_filter(handle, x, dz, z, dw, db, act, alpha, hd->scratch, (size_t)H3D_STATIC_SCRATCH_BYTES, stream);
}
