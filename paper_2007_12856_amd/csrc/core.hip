// Handle, error text and host-side argument validation shared by every entry point.
#include <stdarg.h>

#include <new>

#include "common.h"

namespace h3d {

h3d_status fail(void* handle, h3d_status st, const char* fmt, ...) {
  if (handle) {
    Handle* hd = static_cast<Handle*>(handle);
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(hd->err, sizeof(hd->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

h3d_status check_tensor(void* handle, const h3d_tensor* t, const char* name) {
  if (!handle) return H3D_EINVAL;
  if (!t) return fail(handle, H3D_EINVAL, "%s: NULL descriptor", name);
  if (t->dtype != H3D_F32 && t->dtype != H3D_BF16) return fail(handle, H3D_EINVAL, "%s: bad dtype %d", name, t->dtype);
  if (t->n < 0 || t->c < 0 || t->d < 0 || t->h < 0 || t->w < 0 || t->halo_lo < 0 || t->halo_hi < 0)
    return fail(handle, H3D_EINVAL, "%s: negative extent", name);
  if (t->d_global < 0 || t->d_offset < 0 || t->d_offset + t->d > t->d_global)
    return fail(handle, H3D_EINVAL, "%s: interior [%lld,%lld) not inside the global depth %lld", name,
                (long long)t->d_offset, (long long)(t->d_offset + t->d), (long long)t->d_global);
  int64_t elems = (int64_t)t->n * t->c * (t->halo_lo + t->d + t->halo_hi) * t->h * t->w;
  if (elems > 0 && !t->data) return fail(handle, H3D_EINVAL, "%s: NULL data pointer", name);
  if (elems >= ((int64_t)1 << 40)) return fail(handle, H3D_EINVAL, "%s: tensor too large", name);
  if ((int64_t)t->h * t->w >= ((int64_t)1 << 30)) return fail(handle, H3D_EINVAL, "%s: plane too large", name);
  if (((uintptr_t)t->data) % elt_size(t->dtype)) return fail(handle, H3D_EINVAL, "%s: misaligned data pointer", name);
  if (t->c_stride < 0 || t->n_stride < 0) return fail(handle, H3D_EINVAL, "%s: negative stride", name);
  if (!is_packed(t)) {
    const int64_t run = (int64_t)(t->halo_lo + t->d + t->halo_hi) * t->h * t->w;
    const int64_t cs = t->c_stride ? t->c_stride : run;
    const int64_t ns = t->n_stride ? t->n_stride : cs * t->c;
    if (cs < run || ns < cs * t->c) return fail(handle, H3D_EINVAL, "%s: strides smaller than the run of planes they address", name);
    if (ns >= ((int64_t)1 << 40)) return fail(handle, H3D_EINVAL, "%s: tensor too large", name);
  }
  return H3D_OK;
}

h3d_status check_tensor_packed(void* handle, const h3d_tensor* t, const char* name) {
  H3D_TRY(check_tensor(handle, t, name));
  if (!is_packed(t)) return fail(handle, H3D_EUNSUPPORTED, "%s: strided plane runs are accepted by the convolution passes only", name);
  return H3D_OK;
}

bool same_shard(const h3d_tensor* a, const h3d_tensor* b) {
  return a->n == b->n && a->d == b->d && a->h == b->h && a->w == b->w && a->d_offset == b->d_offset &&
         a->d_global == b->d_global && a->dtype == b->dtype;
}

static inline bool in_volume(const h3d_tensor* t, int64_t p) {
  int64_t g = t->d_offset + p;
  return g >= 0 && g < t->d_global;
}

bool halo_covers(const h3d_tensor* in, int64_t lo, int64_t hi) {
  for (int64_t p = lo; p < hi; ++p) {
    if (!in_volume(in, p)) continue;
    for (int k = -1; k <= 1; ++k) {
      int64_t q = p + k;
      if (in_volume(in, q) && !(q >= -in->halo_lo && q < in->d + in->halo_hi)) return false;
    }
  }
  return true;
}

void note_kernel(void* handle, const char* fmt, ...) {
  if (!handle) return;
  Handle* hd = static_cast<Handle*>(handle);
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(hd->kernel, sizeof(hd->kernel), fmt, ap);
  va_end(ap);
  hd->kernel_noted = true;
}

h3d_status launch_status(void* handle, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(handle, H3D_EHIP, "%s: %s", what, hipGetErrorString(e));
  Handle* hd = static_cast<Handle*>(handle);
  if (hd) {
    if (!hd->kernel_noted) snprintf(hd->kernel, sizeof(hd->kernel), "%s", what);
    hd->kernel_noted = false;          // the next call starts afresh
  }
  return H3D_OK;
}

}  // namespace h3d

using namespace h3d;

extern "C" h3d_status h3d_create(void** handle) {
  if (!handle) return H3D_EINVAL;
  *handle = nullptr;
  Handle* hd = new (std::nothrow) Handle();
  if (!hd) return H3D_EINVAL;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    delete hd;
    return H3D_EHIP;
  }
  hd->device = dev;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, dev) == hipSuccess) hd->num_cu = prop.multiProcessorCount;
  if (static_scratch_init(hd) != H3D_OK) {
    delete hd;
    return H3D_EHIP;
  }
  *handle = hd;
  return H3D_OK;
}

extern "C" h3d_status h3d_destroy(void* handle) {
  if (!handle) return H3D_EINVAL;
  delete static_cast<Handle*>(handle);
  return H3D_OK;
}

extern "C" const char* h3d_last_kernel(void* handle) {
  if (!handle) return "";
  return static_cast<Handle*>(handle)->kernel;
}

extern "C" const char* h3d_last_error(void* handle) {
  if (!handle) return "NULL handle";
  return static_cast<Handle*>(handle)->err;
}
