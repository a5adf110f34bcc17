// Calibration probes for the two rooflines the benchmark reports: what a register-only MFMA loop and a plain
// streaming read reach on the device at hand.  They touch no tensor of the method; a kernel's fraction of the
// published peak is then read beside its fraction of what the chip sustains under the simplest possible load.
#include "common.h"

namespace h3d {

typedef __bf16 pr_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pr_f32x4 __attribute__((ext_vector_type(4)));
typedef float pr_f32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_BLOCKS = 2048, PROBE_THREADS = 256;

// four independent accumulator chains per wavefront, operands fixed in registers
template <int SHAPE>
__global__ void __launch_bounds__(PROBE_THREADS) probe_mfma_kernel(const uint4* __restrict__ seed, float* __restrict__ sink, int iters) {
  const uint4 av = seed[threadIdx.x & 63];
  const pr_bf16x8 A = __builtin_bit_cast(pr_bf16x8, av);
  float s = 0.f;
  if (SHAPE == 0) {
    pr_f32x4 c[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, A, c[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) s += c[j][0] + c[j][1] + c[j][2] + c[j][3];
  } else {
    pr_f32x16 c[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) c[j][r] = 0.f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, A, c[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += c[j][r];
  }
  sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// grid-stride read of 16-byte units, eight loads in flight per lane; the result is stored only if it has a value
// that the data cannot produce by accident, so the loads are kept and nothing is written
__global__ void __launch_bounds__(512) probe_read_kernel(const uint4* __restrict__ p, size_t n16, unsigned* __restrict__ sink) {
  constexpr int UN = 8;
  unsigned acc = 0;
  const size_t stride = (size_t)gridDim.x * 512;
  size_t i = (size_t)blockIdx.x * 512 + threadIdx.x;
  for (; i + (UN - 1) * stride < n16; i += UN * stride) {
    uint4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < UN; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = p[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

}  // namespace h3d

using namespace h3d;

extern "C" size_t h3d_probe_mfma_scratch_bytes(void) { return (size_t)PROBE_BLOCKS * PROBE_THREADS * sizeof(float) + 1024; }

extern "C" h3d_status h3d_probe_mfma_bf16(void* handle, int shape, int iters, void* scratch, size_t scratch_bytes, double* flops,
                                          void* stream) {
  if (!handle) return H3D_EINVAL;
  if ((shape != 0 && shape != 1) || iters < 1 || !scratch || !flops) return fail(handle, H3D_EINVAL, "probe_mfma: bad argument");
  if (scratch_bytes < h3d_probe_mfma_scratch_bytes() || ((uintptr_t)scratch & 15)) return fail(handle, H3D_EWORKSPACE, "probe_mfma: scratch too small or unaligned");
  // operand seed: the first 1024 bytes of the scratch, whatever they hold (the arithmetic result is not used)
  const uint4* seed = (const uint4*)scratch;
  float* sink = (float*)((char*)scratch + 1024);
  if (shape == 0) hipLaunchKernelGGL((probe_mfma_kernel<0>), dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, (hipStream_t)stream, seed, sink, iters);
  else hipLaunchKernelGGL((probe_mfma_kernel<1>), dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, (hipStream_t)stream, seed, sink, iters);
  const double per_mfma = shape == 0 ? 2.0 * 16 * 16 * 32 : 2.0 * 32 * 32 * 16;
  *flops = (double)PROBE_BLOCKS * (PROBE_THREADS / 64) * iters * (shape == 0 ? 4 : 2) * per_mfma;
  return launch_status(handle, "probe_mfma");
}

extern "C" h3d_status h3d_probe_read(void* handle, const void* buf, size_t bytes, void* sink, void* stream) {
  if (!handle) return H3D_EINVAL;
  if (!buf || !sink || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3)) return fail(handle, H3D_EINVAL, "probe_read: NULL or unaligned pointer");
  if (bytes < 16) return H3D_OK;
  const int num_cu = static_cast<Handle*>(handle)->num_cu;
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)(num_cu * 4)), dim3(512), 0, (hipStream_t)stream, (const uint4*)buf, bytes / 16, (unsigned*)sink);
  return launch_status(handle, "probe_read");
}
