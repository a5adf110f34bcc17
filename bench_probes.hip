// Calibration probes for bench.py (NOT part of libh3d and not part of the method): what the device at hand sustains
// under the simplest possible load, so that a kernel's fraction of the published peak can be read beside its fraction
// of a measured ceiling.  Built by __graft_entry__.build() (or by bench.py itself when missing) into
// libbench_probes.so next to this file; plain C entry points, device pointers from the caller, nothing allocated.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 pr_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pr_f32x4 __attribute__((ext_vector_type(4)));
typedef float pr_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned pr_u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_BLOCKS = 2048, PROBE_THREADS = 256;

// independent accumulator chains per wavefront, operands fixed in registers
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

// Streaming read of 16-byte units, UN loads in flight per lane; the result is stored only if it has a value that the
// data cannot produce by accident, so the loads are kept and nothing is written.
// CONTIG = false: grid-stride (lane i of the grid reads units i, i + grid, ...);
// CONTIG = true: every block owns one contiguous piece of the buffer and walks it front to back.
template <int UN, bool CONTIG>
__global__ void __launch_bounds__(256) probe_read_kernel(const pr_u32x4* __restrict__ p, size_t n16, unsigned* __restrict__ sink) {
  unsigned acc = 0;
  size_t i, end, stride;
  if (CONTIG) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    i = (size_t)blockIdx.x * per + threadIdx.x;
    end = (size_t)(blockIdx.x + 1) * per;
    if (end > n16) end = n16;
    stride = 256;
  } else {
    stride = (size_t)gridDim.x * 256;
    i = (size_t)blockIdx.x * 256 + threadIdx.x;
    end = n16;
  }
  for (; i + (UN - 1) * stride < end; i += UN * stride) {
    pr_u32x4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < UN; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < end; i += stride) {
    const pr_u32x4 v = p[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

// streaming write of a constant, and a plain copy, 16-byte units, grid-stride
__global__ void __launch_bounds__(256) probe_write_kernel(uint4* __restrict__ p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  const uint4 v = {1u, 2u, 3u, 4u};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) p[i] = v;
}
template <int UN>
__global__ void __launch_bounds__(256) probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (UN - 1) * stride < n16; i += UN * stride) {
    uint4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < UN; ++u) dst[i + u * stride] = v[u];
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

extern "C" size_t bp_mfma_scratch_bytes(void) { return (size_t)PROBE_BLOCKS * PROBE_THREADS * sizeof(float) + 1024; }

// shape 0: 16x16x32, 1: 32x32x16 (bf16).  *flops (HOST) receives the flop count of the launch.  0 on success.
extern "C" int bp_mfma_bf16(int shape, int iters, void* scratch, size_t scratch_bytes, double* flops, void* stream) {
  if ((shape != 0 && shape != 1) || iters < 1 || !scratch || !flops) return -1;
  if (scratch_bytes < bp_mfma_scratch_bytes() || ((uintptr_t)scratch & 15)) return -3;
  const uint4* seed = (const uint4*)scratch;           // operand seed: the first 1024 bytes, whatever they hold
  float* sink = (float*)((char*)scratch + 1024);
  if (shape == 0) hipLaunchKernelGGL((probe_mfma_kernel<0>), dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, (hipStream_t)stream, seed, sink, iters);
  else hipLaunchKernelGGL((probe_mfma_kernel<1>), dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, (hipStream_t)stream, seed, sink, iters);
  const double per_mfma = shape == 0 ? 2.0 * 16 * 16 * 32 : 2.0 * 32 * 32 * 16;
  *flops = (double)PROBE_BLOCKS * (PROBE_THREADS / 64) * iters * (shape == 0 ? 4 : 2) * per_mfma;
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

// reads `bytes` (whole 16-byte units) of buf once.  blocks: grid size (workgroups of 256 lanes); unroll in {4, 8, 16};
// contig: 0 grid-stride, 1 one contiguous piece per workgroup.
extern "C" int bp_read(const void* buf, size_t bytes, void* sink, int blocks, int unroll, int contig, void* stream) {
  if (!buf || !sink || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3) || blocks < 1) return -1;
  if (bytes < 16) return 0;
  const pr_u32x4* p = (const pr_u32x4*)buf;
  const size_t n16 = bytes / 16;
  unsigned* s = (unsigned*)sink;
  hipStream_t st = (hipStream_t)stream;
#define BP_READ(UN, C) hipLaunchKernelGGL((probe_read_kernel<UN, C>), dim3((unsigned)blocks), dim3(256), 0, st, p, n16, s)
  if (unroll == 4) { if (contig) BP_READ(4, true); else BP_READ(4, false); }
  else if (unroll == 8) { if (contig) BP_READ(8, true); else BP_READ(8, false); }
  else if (unroll == 16) { if (contig) BP_READ(16, true); else BP_READ(16, false); }
  else return -1;
#undef BP_READ
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int bp_write(void* buf, size_t bytes, int blocks, void* stream) {
  if (!buf || ((uintptr_t)buf & 15) || blocks < 1) return -1;
  if (bytes < 16) return 0;
  hipLaunchKernelGGL(probe_write_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)buf, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int bp_copy(const void* src, void* dst, size_t bytes, int blocks, int unroll, void* stream) {
  if (!src || !dst || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15) || blocks < 1) return -1;
  if (bytes < 16) return 0;
  const uint4* s = (const uint4*)src;
  uint4* d = (uint4*)dst;
  if (unroll == 4) hipLaunchKernelGGL((probe_copy_kernel<4>), dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, s, d, bytes / 16);
  else if (unroll == 8) hipLaunchKernelGGL((probe_copy_kernel<8>), dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, s, d, bytes / 16);
  else return -1;
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
