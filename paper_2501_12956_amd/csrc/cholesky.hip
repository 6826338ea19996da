// L = Cholesky(H) or of its preconditioned form (Eq. (10), Remark 3.1,
// Appendix A Eq. (23)-(24)), blocked right-looking, fp32 storage.
//
// Per 64-column panel: (1) the 64 x 64 diagonal block is factored, and the
// factor inverted, by one wavefront; (2) the rows below it are multiplied by
// that inverse (matrix-core GEMM, in place); (3) the trailing lower triangle is
// updated with the fp32 matrix-core GEMM (A A^T form).
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

// Factor the nb x nb diagonal block at (k0, k0) in place and write the inverse of the factor
// (64 x 64, fp32, row-major, identity-padded beyond nb) to `inv`.
//
// Thread (r, g) = (tid / 4, tid % 4) keeps the entries (r, g + 4 i) of ONE 64 x 64 working
// matrix M in registers.  Columns right of the current one hold the not yet factored part
// of A; columns left of it are reused for the right-hand sides of L X = I (column k of L
// is dead once step k has used it and is copied out to LDS).  Step k is a single rank-1
// update  M[r][:] -= L[r][k] * v  for r > k  with  v = ( X[k][0..k-1], 1/L_kk, L[k+1..][k] ),
// one barrier per step (publish buffers are double-buffered).  On a bad pivot the 1-based
// global index of the first one is recorded in *info (if still 0) and the pivot is replaced
// by 1 so that the kernel terminates normally.
// The 64 steps run as 16 iterations of 4 unrolled steps (the unrolled 64 would not fit the
// instruction cache).  The register array is rotated by one after every 4 steps so that
// a[0] always holds the entry of the current column group ik: a[i] is column
// g + 4 ((ik + i) mod 16); positions i >= 16 - ik are columns already factored (they hold
// the inverse), positions 1 .. 15 - ik are columns still to come.
template <int GK>
__device__ inline void potf_step(float (&a)[16], int ik, int r, int g, int nb, int64_t k0,
                                 int* __restrict__ info, float (*vbuf)[NB], float* __restrict__ piv,
                                 float (*Lout)[NB + 1]) {
  constexpr int bf = GK & 1;
  const int K = 4 * ik + GK;
  // Publish the raw vector  v = ( M[K][c] for c < K, 1 at c == K, M[c][K] for c > K )  in
  // the readers' register order: entry c at [(c & 3) * 16 + ((c / 4 - ik) mod 16)], i.e.
  // thread (., g) finds the entries of its 16 registers at [16 g .. 16 g + 15].
  if (r == K) {
#pragma unroll
    for (int i = 1; i < 16; ++i)
      if (i >= 16 - ik) vbuf[bf][g * 16 + i] = a[i];       // columns already factored
    if (g < GK) vbuf[bf][g * 16] = a[0];
    if (g == GK) {
      vbuf[bf][g * 16] = 1.f;
      piv[bf] = a[0];
    }
  } else if (r > K && g == GK) {
    vbuf[bf][(r & 3) * 16 + (((r >> 2) - ik) & 15)] = a[0];
  }
  __syncthreads();
  float d = piv[bf];
  if (!(d > 0.f) || !(d < 3.0e38f)) {
    if (r == 0 && g == 0 && K < nb) atomicCAS(info, 0, (int)(k0 + K + 1));
    d = 1.f;
  }
  const float sd = sqrtf(d);
  const float rs = 1.f / sd;
  const float lraw = vbuf[bf][(r & 3) * 16 + (((r >> 2) - ik) & 15)];   // M[r][K] for r > K
  if (g == GK) Lout[r][K] = (r == K) ? sd : ((r > K) ? lraw * rs : 0.f);
  // rows r > K: M[r][c] -= L[r][K] * (v[c] / L_KK)  (the entry at c == K starts from 0);
  // row K: M[K][c] = v[c] / L_KK (its part of the inverse is final); rows r < K: unchanged.
  // Entries above the diagonal receive harmless finite values that nothing reads.
  const float coef = (r > K) ? -(lraw * rs) * rs : ((r == K) ? rs : 0.f);
  const bool zero_row = (r == K);
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const float4 vv = *reinterpret_cast<const float4*>(&vbuf[bf][g * 16 + 4 * i4]);
    const float ve[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = 4 * i4 + e;
      const bool zero_in = zero_row || (i == 0 && g == GK);
      a[i] = fmaf(coef, ve[e], zero_in ? 0.f : a[i]);
    }
  }
}

__global__ __launch_bounds__(256) void potf2_inv_kernel(float* __restrict__ L, int64_t ldl,
                                                        int64_t k0, int nb, int* __restrict__ info,
                                                        float* __restrict__ inv) {
  __shared__ float Lout[NB][NB + 1];
  __shared__ __attribute__((aligned(16))) float vbuf[2][NB];
  __shared__ float piv[2];
  const int tid = threadIdx.x, r = tid >> 2, g = tid & 3;
  // coalesced load through LDS (identity padding beyond nb, strict upper part zero)
  for (int e = tid; e < NB * NB; e += 256) {
    const int rr = e >> 6, cc = e & 63;
    float v = (rr == cc) ? 1.f : 0.f;
    if (rr < nb && cc < nb) v = (cc <= rr) ? L[(k0 + rr) * ldl + k0 + cc] : 0.f;
    Lout[rr][cc] = v;
  }
  __syncthreads();
  float a[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) a[i] = Lout[r][g + 4 * i];
  __syncthreads();
  for (int ik = 0; ik < 16; ++ik) {
    potf_step<0>(a, ik, r, g, nb, k0, info, vbuf, piv, Lout);
    potf_step<1>(a, ik, r, g, nb, k0, info, vbuf, piv, Lout);
    potf_step<2>(a, ik, r, g, nb, k0, info, vbuf, piv, Lout);
    potf_step<3>(a, ik, r, g, nb, k0, info, vbuf, piv, Lout);
    const float t0 = a[0];
#pragma unroll
    for (int i = 0; i < 15; ++i) a[i] = a[i + 1];
    a[15] = t0;
  }
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int rr = e >> 6, cc = e & 63;
    if (rr < nb && cc <= rr) L[(k0 + rr) * ldl + k0 + cc] = Lout[rr][cc];
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = g + 4 * i;
    inv[r * NB + c] = (c <= r) ? a[i] : 0.f;
  }
}

}  // namespace

size_t cholesky_scratch_bytes(int64_t n) {
  return kAlign + align_up((size_t)n * sizeof(float)) + align_up((size_t)NB * NB * sizeof(float));
}

hipError_t launch_cholesky(hipStream_t s, const float* H, int64_t n, int64_t ldh, int precond,
                           float lambda, float* L, int64_t ldl, int* info_dev) {
  // info_dev points at scratch: [int info][pad to 256][float delta[n]][float inv[64 x 64]]
  float* delta = reinterpret_cast<float*>(reinterpret_cast<char*>(info_dev) + kAlign);
  float* inv = reinterpret_cast<float*>(reinterpret_cast<char*>(delta) + align_up((size_t)n * sizeof(float)));
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
    hipLaunchKernelGGL(potf2_inv_kernel, dim3(1), dim3(256), 0, s, L, ldl, k0, nb, info_dev, inv);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int64_t rem = n - k0 - nb;
    if (rem <= 0) break;
    float* A21 = L + (k0 + nb) * ldl + k0;
    float* A22 = L + (k0 + nb) * ldl + (k0 + nb);
    // panel solve as a product with the inverse of the diagonal factor, in place: each
    // workgroup of the GEMM reads all of its rows of A21 before it writes them
    e = launch_gemm_f32(s, /*transb=*/1, /*lower_only=*/0, rem, nb, nb, 1.f, A21, ldl, inv, NB, 0.f,
                        A21, ldl);
    if (e != hipSuccess) return e;
    e = launch_gemm_f32(s, /*transb=*/1, /*lower_only=*/1, rem, rem, nb, -1.f, A21, ldl, A21, ldl,
                        1.f, A22, ldl);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ganq
