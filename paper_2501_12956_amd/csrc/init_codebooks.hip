// T^0: initial per-row codebooks (input of Algorithm 1), built from per-row
// quantiles of W.  One workgroup per row sorts the row in LDS (bitonic network,
// padded with +inf to a power of two) and interpolates the C requested order
// statistics.  Also: fp16 -> fp32 conversion of W for the fp32 solve.
#include "ganq_internal.h"

namespace ganq {
namespace {

template <typename TW>
__global__ __launch_bounds__(1024) void init_codebooks_kernel(const TW* __restrict__ W, int64_t n,
                                                              int64_t ldw, int npow2, int C,
                                                              int mode, float* __restrict__ T) {
  extern __shared__ float srt[];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  for (int e = tid; e < npow2; e += 1024)
    srt[e] = (e < n) ? (float)W[row * ldw + e] : __builtin_huge_valf();
  __syncthreads();
  bitonic_sort_lds_1024(srt, npow2, tid);
  if (tid < C) {
    const int s = tid;
    double val;
    if (mode == GANQ_INIT_MINMAX_GRID) {
      const double lo = srt[0], hi = srt[n - 1];
      const double frac = (C > 1) ? (double)s / (double)(C - 1) : 0.0;
      val = lo + frac * (hi - lo);
    } else {
      double q;
      if (mode == GANQ_INIT_QUANTILE_MID)
        q = ((double)s + 0.5) / (double)C;
      else
        q = (C > 1) ? (double)s / (double)(C - 1) : 0.5;
      const double h = q * (double)(n - 1);
      int64_t lo = (int64_t)floor(h);
      if (lo > n - 1) lo = n - 1;
      const int64_t hi = (lo + 1 < n) ? lo + 1 : n - 1;
      const double a = srt[lo], b = srt[hi];
      val = a + (h - (double)lo) * (b - a);
    }
    T[row * C + s] = (float)val;
  }
}

__global__ __launch_bounds__(256) void convert_f16_f32_kernel(const _Float16* __restrict__ src,
                                                              int64_t cols, int64_t ld_src,
                                                              float* __restrict__ dst,
                                                              int64_t ld_dst) {
  const int64_t r = blockIdx.y;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < cols; c += (int64_t)gridDim.x * 256)
    dst[r * ld_dst + c] = (float)src[r * ld_src + c];
}

}  // namespace

hipError_t launch_init_codebooks(hipStream_t s, const void* W, int w_is_f16, int64_t m, int64_t n,
                                 int64_t ldw, int nbits, int mode, float* T) {
  int npow2 = 1;
  while (npow2 < n) npow2 <<= 1;
  const size_t shmem = (size_t)npow2 * sizeof(float);
  const int C = 1 << nbits;
  hipError_t e;
  if (w_is_f16) {
    auto kern = init_codebooks_kernel<_Float16>;
    if (shmem > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)shmem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)m), dim3(1024), shmem, s, (const _Float16*)W, n, ldw,
                       npow2, C, mode, T);
  } else {
    auto kern = init_codebooks_kernel<float>;
    if (shmem > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)shmem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)m), dim3(1024), shmem, s, (const float*)W, n, ldw,
                       npow2, C, mode, T);
  }
  return hipGetLastError();
}

hipError_t launch_convert_f16_f32(hipStream_t s, const _Float16* src, int64_t rows, int64_t cols,
                                  int64_t ld_src, float* dst, int64_t ld_dst) {
  dim3 grid((unsigned)((cols + 1023) / 1024 > 0 ? (cols + 1023) / 1024 : 1), (unsigned)rows);
  hipLaunchKernelGGL(convert_f16_f32_kernel, grid, dim3(256), 0, s, src, cols, ld_src, dst, ld_dst);
  return hipGetLastError();
}

}  // namespace ganq
