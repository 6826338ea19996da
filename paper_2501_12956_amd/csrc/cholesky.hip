// L = Cholesky(H) or of its preconditioned form (Eq. (10), Remark 3.1,
// Appendix A Eq. (23)-(24)), blocked right-looking, fp32 storage.
//
// Per 64-column panel: (1) the 64 x 64 diagonal block is factored by one
// workgroup in LDS in float64; (2) the rows below it are solved against the
// block (one thread per row, the block broadcast from LDS); (3) the trailing
// lower triangle is updated with the fp32 matrix-core GEMM (A A^T form).
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int NB = 64;

__global__ void fill_i32_kernel(int* p, int v) { *p = v; }

// L <- lower triangle of H (+ preconditioner on the diagonal), strict upper zeroed.
// delta (if used) must already hold the diagonal offsets.
__global__ __launch_bounds__(256) void copy_lower_kernel(const float* __restrict__ H, int64_t n,
                                                         int64_t ldh, float* __restrict__ L,
                                                         int64_t ldl, int precond, float lambda,
                                                         const float* __restrict__ delta) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i = blockIdx.y;
  if (j >= n) return;
  float v = 0.f;
  if (j <= i) {
    v = H[i * ldh + j];
    if (j == i) {
      if (precond == GANQ_PRECOND_LAMBDA) v += lambda;
      if (precond == GANQ_PRECOND_DIAGDOM) v += delta[i];
    }
  }
  L[i * ldl + j] = v;
}

// delta_i = max(sum_j |H_ij| - 2 H_ii, 1e-8), Appendix A Eq. (23); one workgroup per row.
__global__ __launch_bounds__(256) void diagdom_delta_kernel(const float* __restrict__ H, int64_t n,
                                                            int64_t ldh, float* __restrict__ delta) {
  const int64_t i = blockIdx.x;
  double s = 0.0;
  for (int64_t j = threadIdx.x; j < n; j += 256) s += fabs((double)H[i * ldh + j]);
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double d = red[0] - 2.0 * (double)H[i * ldh + i];
    delta[i] = (float)(d > 1e-8 ? d : 1e-8);
  }
}

// Factor the nb x nb diagonal block at (k0, k0) in place.  On a bad pivot the
// 1-based global index of the first one is recorded in *info (if still 0) and
// the pivot is replaced by 1 so that the kernel terminates normally.
__global__ __launch_bounds__(256) void potf2_kernel(float* __restrict__ L, int64_t ldl, int64_t k0,
                                                    int nb, int* __restrict__ info) {
  __shared__ double A[NB][NB + 1];
  const int tid = threadIdx.x;
  for (int e = tid; e < nb * nb; e += 256) {
    const int r = e / nb, c = e % nb;
    A[r][c] = (c <= r) ? (double)L[(k0 + r) * ldl + k0 + c] : 0.0;
  }
  __syncthreads();
  for (int k = 0; k < nb; ++k) {
    double d = A[k][k];
    const bool bad = !(d > 0.0) || !(d < 1.79e308);
    if (bad) {
      if (tid == 0) atomicCAS(info, 0, (int)(k0 + k + 1));
      d = 1.0;
    }
    const double s = sqrt(d);
    __syncthreads();
    if (tid == 0) A[k][k] = s;
    for (int r = k + 1 + tid; r < nb; r += 256) A[r][k] /= s;
    __syncthreads();
    // trailing update of the lower triangle: A[r][c] -= A[r][k] A[c][k], k < c <= r
    const int rem = nb - k - 1;
    for (int e = tid; e < rem * rem; e += 256) {
      const int r = k + 1 + e / rem, c = k + 1 + e % rem;
      if (c <= r) A[r][c] -= A[r][k] * A[c][k];
    }
    __syncthreads();
  }
  for (int e = tid; e < nb * nb; e += 256) {
    const int r = e / nb, c = e % nb;
    if (c <= r) L[(k0 + r) * ldl + k0 + c] = (float)A[r][c];
  }
}

// Rows [r0, n) of the panel: X <- X * L11^{-T}, L11 the factored nb x nb block at (k0, k0).
__global__ __launch_bounds__(64) void trsm_kernel(float* __restrict__ L, int64_t ldl, int64_t n,
                                                  int64_t k0, int nb) {
  __shared__ float D[NB][NB + 1];     // L11, row-major
  __shared__ float Xs[NB][NB + 1];    // 64 rows of the panel
  const int tid = threadIdx.x;
  const int64_t r0 = k0 + nb + (int64_t)blockIdx.x * NB;
  for (int r = 0; r < nb; ++r) D[r][tid] = (tid < nb && tid <= r) ? L[(k0 + r) * ldl + k0 + tid] : 0.f;
  for (int r = 0; r < NB; ++r)
    Xs[r][tid] = (r0 + r < n && tid < nb) ? L[(r0 + r) * ldl + k0 + tid] : 0.f;
  __syncthreads();
  float x[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) x[c] = Xs[tid][c];
#pragma unroll
  for (int c = 0; c < NB; ++c) {
    if (c < nb) {
      float s = x[c];
#pragma unroll
      for (int q = 0; q < c; ++q) s -= x[q] * D[c][q];
      x[c] = s / D[c][c];
    }
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < NB; ++c) Xs[tid][c] = x[c];
  __syncthreads();
  for (int r = 0; r < NB; ++r)
    if (r0 + r < n && tid < nb) L[(r0 + r) * ldl + k0 + tid] = Xs[r][tid];
}

}  // namespace

size_t cholesky_scratch_bytes(int64_t n) { return align_up((size_t)n * sizeof(float)) + kAlign; }

hipError_t launch_cholesky(hipStream_t s, const float* H, int64_t n, int64_t ldh, int precond,
                           float lambda, float* L, int64_t ldl, int* info_dev) {
  // info_dev points at scratch: [int info][pad to 256][float delta[n]]
  float* delta = reinterpret_cast<float*>(reinterpret_cast<char*>(info_dev) + kAlign);
  hipError_t e;
  hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(1), 0, s, info_dev, 0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (precond == GANQ_PRECOND_DIAGDOM) {
    hipLaunchKernelGGL(diagdom_delta_kernel, dim3((unsigned)n), dim3(256), 0, s, H, n, ldh, delta);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  hipLaunchKernelGGL(copy_lower_kernel, dim3((unsigned)ceil_div(n, 256), (unsigned)n), dim3(256),
                     0, s, H, n, ldh, L, ldl, precond, lambda, delta);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  for (int64_t k0 = 0; k0 < n; k0 += NB) {
    const int nb = (int)((n - k0 < NB) ? n - k0 : NB);
    hipLaunchKernelGGL(potf2_kernel, dim3(1), dim3(256), 0, s, L, ldl, k0, nb, info_dev);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int64_t rem = n - k0 - nb;
    if (rem <= 0) break;
    hipLaunchKernelGGL(trsm_kernel, dim3((unsigned)ceil_div(rem, NB)), dim3(64), 0, s, L, ldl, n,
                       k0, nb);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    float* A21 = L + (k0 + nb) * ldl + k0;
    float* A22 = L + (k0 + nb) * ldl + (k0 + nb);
    e = launch_gemm_f32(s, /*transb=*/1, /*lower_only=*/1, rem, rem, nb, -1.f, A21, ldl, A21, ldl,
                        1.f, A22, ldl);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ganq
