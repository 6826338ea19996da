// fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32).
//
// Serves the steps of the GANQ layer solver that need exact fp32 products: the
// trailing updates of the blocked Cholesky factorisation (Eq. (10)) and
// H = X X^T for fp32 activations (Eq. (9)).
//
// Workgroup tile 128 x 128 x 16, 256 threads = 4 wavefronts in a 2 x 2 grid,
// each wavefront owning a 64 x 64 sub-tile as 2 x 2 MFMA tiles of 32 x 32.
// Operands are staged k-major in LDS so that one MFMA operand fetch is one
// conflict-free ds_read_b32 per lane; the next k-slab is prefetched from
// global memory into registers while the current one is multiplied.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int BM = 128, BN = 128, BK = 16, PAD = 4;

struct Frag {
  float v[4];
};

// Four consecutive elements of a row of a row-major matrix, zero-filled outside
// [0, rows) x [0, cols).  `vec` says the fast 16-byte path is legal.
__device__ inline Frag load_row4(const float* __restrict__ base, int64_t row, int64_t col,
                                 int64_t rows, int64_t cols, int64_t ld, bool vec) {
  Frag f;
  if (row < rows && vec && col + 3 < cols) {
    float4 q = *reinterpret_cast<const float4*>(base + row * ld + col);
    f.v[0] = q.x; f.v[1] = q.y; f.v[2] = q.z; f.v[3] = q.w;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      f.v[i] = (row < rows && col + i < cols) ? base[row * ld + col + i] : 0.f;
  }
  return f;
}

template <int TRANSB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int lower_only, int64_t M, int64_t N,
                                                       int64_t K, float alpha,
                                                       const float* __restrict__ A, int64_t lda,
                                                       const float* __restrict__ B, int64_t ldb,
                                                       float beta, float* __restrict__ C,
                                                       int64_t ldc, int vecA, int vecB) {
  const int bm = blockIdx.y, bn = blockIdx.x;
  if (lower_only && bn > bm) return;
  __shared__ float As[BK][BM + PAD];
  __shared__ float Bs[BK][BN + PAD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // global -> register staging
  Frag ra[2], rb[2];
  const int a_row = tid >> 2, a_k4 = (tid & 3) * 4;      // A (and B when TRANSB): rows x k
  const int b_k = tid >> 5, b_n4 = (tid & 31) * 4;       // B when !TRANSB: k x cols

  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
      ra[ps] = load_row4(A, m0 + a_row + 64 * ps, k0 + a_k4, M, K, lda, vecA);
      if (TRANSB)
        rb[ps] = load_row4(B, n0 + a_row + 64 * ps, k0 + a_k4, N, K, ldb, vecB);
      else
        rb[ps] = load_row4(B, k0 + b_k + 8 * ps, n0 + b_n4, K, N, ldb, vecB);
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
#pragma unroll
      for (int i = 0; i < 4; ++i) As[a_k4 + i][a_row + 64 * ps] = ra[ps].v[i];
      if (TRANSB) {
#pragma unroll
        for (int i = 0; i < 4; ++i) Bs[a_k4 + i][a_row + 64 * ps] = rb[ps].v[i];
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) Bs[b_k + 8 * ps][b_n4 + i] = rb[ps].v[i];
      }
    }
  };

  fetch(0);
  for (int64_t k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();
    stage();
    __syncthreads();
    if (k0 + BK < K) fetch(k0 + BK);
    const int kh = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float a0 = As[kk + kh][wr * 64 + l32];
      float a1 = As[kk + kh][wr * 64 + 32 + l32];
      float b0 = Bs[kk + kh][wc * 64 + l32];
      float b1 = Bs[kk + kh][wc * 64 + 32 + l32];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
  }

  const int kh = lane >> 5, l32 = lane & 31;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t col = n0 + wc * 64 + j * 32 + l32;
      if (col >= N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wr * 64 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
        if (row >= M) continue;
        if (lower_only && col > row) continue;
        float* cp = C + row * ldc + col;
        float r = alpha * acc[i][j][v];
        if (beta != 0.f) r += beta * (*cp);
        *cp = r;
      }
    }
}

}  // namespace

hipError_t launch_gemm_f32(hipStream_t s, int transb, int lower_only, int64_t M, int64_t N,
                           int64_t K, float alpha, const float* A, int64_t lda, const float* B,
                           int64_t ldb, float beta, float* C, int64_t ldc) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((unsigned)ceil_div(N, BN), (unsigned)ceil_div(M, BM));
  int vecA = (lda % 4 == 0) && (((uintptr_t)A) % 16 == 0);
  int vecB = (ldb % 4 == 0) && (((uintptr_t)B) % 16 == 0);
  if (transb)
    hipLaunchKernelGGL(gemm_f32_kernel<1>, grid, dim3(256), 0, s, lower_only, M, N, K, alpha, A,
                       lda, B, ldb, beta, C, ldc, vecA, vecB);
  else
    hipLaunchKernelGGL(gemm_f32_kernel<0>, grid, dim3(256), 0, s, lower_only, M, N, K, alpha, A,
                       lda, B, ldb, beta, C, ldc, vecA, vecB);
  return hipGetLastError();
}

}  // namespace ganq
