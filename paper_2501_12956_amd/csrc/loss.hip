// Objective of Eq. (1) in the form of Eq. (9): sum_i E_i H E_i^T, E = W - T[Q].
// E is formed here, F = E H comes from the split-fp16 matrix-core GEMM, and the
// row values sum_j F_ij E_ij are reduced per row in float64 and then over rows.
#include "ganq_internal.h"

namespace ganq {
namespace {

__global__ __launch_bounds__(256) void residual_kernel(const float* __restrict__ W, int64_t n,
                                                       int64_t ldw, const float* __restrict__ T,
                                                       const uint8_t* __restrict__ Q, int64_t ldq,
                                                       int C, float* __restrict__ E, int64_t lde) {
  const int64_t i = blockIdx.y;
  __shared__ float tr[16];
  if ((int)threadIdx.x < C) tr[threadIdx.x] = T[i * C + threadIdx.x];
  __syncthreads();
  for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < n; j += (int64_t)gridDim.x * 256)
    E[i * lde + j] = W[i * ldw + j] - tr[Q[i * ldq + j] & (C - 1)];
}

__global__ __launch_bounds__(256) void rowdot_kernel(const float* __restrict__ F, int64_t ldf,
                                                     const float* __restrict__ E, int64_t lde,
                                                     int64_t n, float* __restrict__ row_loss) {
  const int64_t i = blockIdx.x;
  double s = 0.0;
  for (int64_t j = threadIdx.x; j < n; j += 256) s += (double)F[i * ldf + j] * (double)E[i * lde + j];
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) row_loss[i] = (float)red[0];
}

__global__ __launch_bounds__(256) void sum_f64_kernel(const float* __restrict__ v, int64_t m,
                                                      double* __restrict__ out) {
  double s = 0.0;
  for (int64_t i = threadIdx.x; i < m; i += 256) s += (double)v[i];
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0];
}

}  // namespace

size_t loss_scratch_bytes(int64_t m, int64_t n) {
  // E, F (m x n fp32 each), row values, one double
  return 2 * align_up((size_t)m * (size_t)n * sizeof(float)) + align_up((size_t)m * sizeof(float)) +
         kAlign;
}

hipError_t launch_residual(hipStream_t s, const float* W, int64_t m, int64_t n, int64_t ldw,
                           const float* T, const uint8_t* Q, int64_t ldq, int nbits, float* E,
                           int64_t lde) {
  int64_t gx = ceil_div(n, 1024);
  if (gx < 1) gx = 1;
  hipLaunchKernelGGL(residual_kernel, dim3((unsigned)gx, (unsigned)m), dim3(256), 0, s, W, n, ldw, T,
                     Q, ldq, 1 << nbits, E, lde);
  return hipGetLastError();
}

hipError_t launch_rowdot(hipStream_t s, const float* F, int64_t ldf, const float* E, int64_t lde,
                         int64_t m, int64_t n, float* row_loss) {
  hipLaunchKernelGGL(rowdot_kernel, dim3((unsigned)m), dim3(256), 0, s, F, ldf, E, lde, n, row_loss);
  return hipGetLastError();
}

hipError_t launch_sum_f64(hipStream_t s, const float* v, int64_t m, double* out_dev) {
  hipLaunchKernelGGL(sum_f64_kernel, dim3(1), dim3(256), 0, s, v, m, out_dev);
  return hipGetLastError();
}

}  // namespace ganq
