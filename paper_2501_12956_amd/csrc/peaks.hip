// On-box peak probes (measurement aid, not part of the method): register-resident loops of the
// three matrix-core instructions the library's kernels are built on, and a plain device copy.
// The benchmark reports roofline fractions against the published peaks and against these.
#include "ganq_internal.h"

namespace ganq {
namespace {

typedef int intx16 __attribute__((ext_vector_type(16)));

// 4 independent accumulators per wavefront, 2 wavefronts per SIMD: back-to-back issue
constexpr int kProbeIters = 2048;

__global__ __launch_bounds__(512) void probe_f16_kernel(float* out, int iters) {
  half8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)(0.001f * (threadIdx.x & 7));
    b[i] = (_Float16)(0.002f * (threadIdx.x & 3));
  }
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[t], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) s += acc[t][0];
  if (s == 12345.678f) out[0] = s;       // keeps the loop alive; never true
}

__global__ __launch_bounds__(512) void probe_f32_kernel(float* out, int iters) {
  const float a = 0.001f * (threadIdx.x & 7), b = 0.002f * (threadIdx.x & 3);
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[t], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) s += acc[t][0];
  if (s == 12345.678f) out[0] = s;
}

__global__ __launch_bounds__(512) void probe_i8_kernel(float* out, int iters) {
  int4v a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = 0x01020304 * (int)(threadIdx.x & 3);
    b[i] = 0x01000100 * (int)(threadIdx.x & 1);
  }
  intx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[t], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int t = 0; t < 4; ++t) s += acc[t][0];
  if (s == 0x7fffffff) out[0] = (float)s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace

// which: 0 fp16 32x32x16, 1 fp32 32x32x2, 2 int8 32x32x32 (each returns operations per launch in
// *ops), 3 copy of `bytes` from buf to buf + bytes (returns bytes moved, read + write)
hipError_t launch_peak_probe(hipStream_t s, int which, void* buf, size_t bytes, double* ops) {
  const int wgs = 256 * 4;                       // four workgroups of 8 wavefronts per compute unit in turn
  const double waves = (double)wgs * 8.0;
  switch (which) {
    case 0:
      hipLaunchKernelGGL(probe_f16_kernel, dim3(wgs), dim3(512), 0, s, (float*)buf, kProbeIters);
      *ops = waves * kProbeIters * 4.0 * (2.0 * 32 * 32 * 16);
      break;
    case 1:
      hipLaunchKernelGGL(probe_f32_kernel, dim3(wgs), dim3(512), 0, s, (float*)buf, kProbeIters);
      *ops = waves * kProbeIters * 4.0 * (2.0 * 32 * 32 * 2);
      break;
    case 2:
      hipLaunchKernelGGL(probe_i8_kernel, dim3(wgs), dim3(512), 0, s, (float*)buf, kProbeIters);
      *ops = waves * kProbeIters * 4.0 * (2.0 * 32 * 32 * 32);
      break;
    default: {
      const int64_t n16 = (int64_t)(bytes / 16);
      hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, s, (const uint4*)buf,
                         (uint4*)((char*)buf + bytes), n16);
      *ops = 2.0 * (double)n16 * 16.0;
      break;
    }
  }
  return hipGetLastError();
}

}  // namespace ganq
