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


// ---- C(lower) -= A A^T for A of exactly 256 columns: the trailing update of the blocked Cholesky ----
//
// The general kernel above stages 16 columns at a time and leans on several resident workgroups
// to hide the latency of each step; with K = 256 it spends most of its time waiting.  Here the
// whole K extent goes through LDS in four stages of 64 columns, two in flight: operand rows come
// straight from global memory into LDS (buffer_load ... lds, 16 bytes per lane, 4 rows of 256 bytes
// per instruction), the 16-byte chunks of a row stored at position chunk ^ (row & 15) so that a
// 16-byte fragment read of 16 consecutive rows touches every bank once.  A lane's 16-byte read
// supplies four MFMAs: lanes 0..31 hold columns 8g..8g+3 of their row, lanes 32..63 columns
// 8g+4..8g+7, and v_mfma_f32_32x32x2_f32 number t multiplies element t of both (the order in which
// the 256 products of an entry are summed does not matter).  Workgroup tile 128 x 128, four
// wavefronts of 64 x 64; only tiles on or below the diagonal are launched.  C is read at the start
// and the difference written at the end.
constexpr int SK = 256;            // columns of A
constexpr int SKS = 64;            // columns per LDS stage
constexpr int SROWB = SKS * 4;     // bytes per LDS row
constexpr int STILEB = 128 * SROWB;
constexpr int SSTAGEB = 2 * STILEB;
constexpr int SYRK_LDS = 2 * SSTAGEB;

__global__ __launch_bounds__(256) void syrk_f32_kernel(int64_t M, const float* __restrict__ A, int64_t lda,
                                                       float* __restrict__ C, int64_t ldc) {
  // tile t of the lower triangle: row bm, column bn <= bm
  const int t = blockIdx.x;
  int bm = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
  while ((bm + 1) * (bm + 2) / 2 <= t) ++bm;
  while (bm * (bm + 1) / 2 > t) --bm;
  const int bn = t - bm * (bm + 1) / 2;
  const int64_t m0 = (int64_t)bm * 128, n0 = (int64_t)bn * 128;

  extern __shared__ __attribute__((aligned(16))) unsigned char ssm[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)ssm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 1, wc = wave & 1;
  const int kh = lane >> 5, l32 = lane & 31;

  auto make = [&](int64_t r0) {
    const int64_t rows = (M - r0 < 128) ? M - r0 : 128;
    const uint64_t ad = (uint64_t)(uintptr_t)(A + r0 * lda);
    int4v r;
    r[0] = (int)(uint32_t)ad;
    r[1] = (int)(uint32_t)((ad >> 32) & 0xffffu);
    r[2] = (int)(uint32_t)(((rows - 1) * lda + SK) * 4);      // rows past the matrix read as zero
    r[3] = 0x00020000;
    return r;
  };
  const int4v rsA = make(m0), rsB = make(n0);

  // one direct load: lane -> row lane / 16 of a group of 4 rows, LDS chunk position lane % 16
  const int dr = lane >> 4, dp = lane & 15;
  uint32_t voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = (wave + 4 * j) * 4 + dr;                 // 32 groups of 4 rows over 4 wavefronts
    voff[j] = (uint32_t)(((int64_t)row * lda + ((dp ^ (row & 15)) * 4)) * 4);
  }
  auto issue = [&](int ks, int st) {
    const uint32_t soff = (uint32_t)(ks * SKS * 4);
    const uint32_t sb = lds0 + st * SSTAGEB;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      load16_to_lds(rsA, sb + (wave + 4 * j) * 1024, voff[j], soff);
      load16_to_lds(rsB, sb + STILEB + (wave + 4 * j) * 1024, voff[j], soff);
    }
  };

  issue(0, 0);
  // the tile of C, fetched while the first operands are on their way.  A tile that lies wholly
  // inside the matrix and strictly below the diagonal (most of them) needs no per-element tests.
  const bool full = (m0 + 128 <= M) && (bn < bm);
  floatx16 cin[2][2];
  if (full) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float* __restrict__ cp = C + (m0 + wr * 64 + i * 32 + kh * 4) * ldc + n0 + wc * 64 + j * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) cin[i][j][v] = cp[((v >> 2) * 8 + (v & 3)) * ldc];
      }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int64_t col = n0 + wc * 64 + j * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t row = m0 + wr * 64 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
          cin[i][j][v] = (row < M && col <= row) ? C[row * ldc + col] : 0.f;
        }
      }
  }
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  int st = 0;
#pragma unroll 1
  for (int ks = 0; ks < SK / SKS; ++ks) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (ks + 1 < SK / SKS) issue(ks + 1, st ^ 1);
    const unsigned char* As = ssm + st * SSTAGEB;
    const unsigned char* Bs = As + STILEB;
#pragma unroll
    for (int g = 0; g < SKS / 8; ++g) {
      floatx4 af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = wr * 64 + i * 32 + l32;
        af[i] = *reinterpret_cast<const floatx4*>(As + row * SROWB + (((2 * g + kh) ^ (row & 15)) << 4));
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = wc * 64 + j * 32 + l32;
        bf[j] = *reinterpret_cast<const floatx4*>(Bs + row * SROWB + (((2 * g + kh) ^ (row & 15)) << 4));
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][e], bf[j][e], acc[i][j], 0, 0, 0);
    }
    st ^= 1;
  }

  if (full) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float* __restrict__ cp = C + (m0 + wr * 64 + i * 32 + kh * 4) * ldc + n0 + wc * 64 + j * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) cp[((v >> 2) * 8 + (v & 3)) * ldc] = cin[i][j][v] - acc[i][j][v];
      }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int64_t col = n0 + wc * 64 + j * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t row = m0 + wr * 64 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
          if (row < M && col <= row) C[row * ldc + col] = cin[i][j][v] - acc[i][j][v];
        }
      }
  }
}

}  // namespace

// C (M x M, lower triangle) -= A A^T with A of M x 256; needs lda % 4 == 0 and a 16-byte aligned A
// (the caller falls back to launch_gemm_f32 otherwise).
hipError_t launch_syrk256_f32(hipStream_t s, int64_t M, const float* A, int64_t lda, float* C, int64_t ldc) {
  if (M <= 0) return hipSuccess;
  if ((lda % 4) != 0 || (((uintptr_t)A) % 16) != 0 || 128 * lda * 4 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
  static std::atomic<uint64_t> lds_set{0};
  const hipError_t ea = ensure_dynamic_lds((const void*)syrk_f32_kernel, SYRK_LDS, lds_set);
  if (ea != hipSuccess) return ea;
  const int64_t nt = ceil_div(M, 128);
  hipLaunchKernelGGL(syrk_f32_kernel, dim3((unsigned)(nt * (nt + 1) / 2)), dim3(256), SYRK_LDS, s, M, A, lda, C, ldc);
  return hipGetLastError();
}

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
