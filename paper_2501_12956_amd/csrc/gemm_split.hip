// C = A B^T for fp32 A (M x K) and B (N x K) on the fp16 matrix cores with fp32 accuracy to
// about 2^-21: each operand is scaled by a power of two (largest magnitude near 2^14) and
// split into two fp16 pieces, x = hi + lo with |lo| <= 2^-11 |hi| (22 significant bits), and
//     A B^T = Ahi Bhi^T + Ahi Blo^T + Alo Bhi^T        (+ Alo Blo^T, below 2^-22, dropped)
// is accumulated in fp32 by v_mfma_f32_32x32x16_f16 as ONE product over a K axis three times
// as long.  Used for G = W H (T-update, Eq. (7): H is symmetric, so its rows serve as the
// rows of B) and for F = E H of the objective (Eq. (9)); both have a relative tolerance of
// 1e-4 downstream.  The Cholesky factorization keeps the fp32 GEMM.
//
// The product kernel is the H = X X^T kernel's skeleton: 256 x 256 tiles, 8 wavefronts of
// 128 x 64, operand tiles loaded straight into LDS (buffer_load ... lds) in 64-wide K steps
// with XOR-permuted 16-byte chunks, two stages, one barrier per step.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int GT = 256;          // output tile
constexpr int GK = 64;           // k per LDS stage: one 128-byte line per row
constexpr int GROWB = GK * 2;
constexpr int GTILEB = GT * GROWB;
constexpr int GSTAGEB = 2 * GTILEB;
constexpr int GNW = 8;
constexpr int GDPW = (GT / 8) / GNW;

__global__ void fill_u32_kernel(unsigned* p, int count, unsigned v) {
  if ((int)threadIdx.x < count) p[threadIdx.x] = v;
}

// amax[0] = bit pattern of max |x| over the matrix (non-negative floats order like uints)
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ X, int64_t rows, int64_t cols,
                                                     int64_t ld, unsigned* __restrict__ amax) {
  __shared__ float red[256];
  float mx = 0.f;
  for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
    const float* __restrict__ xr = X + r * ld;
    // eight loads in flight per thread; the index is clamped so that they stay unconditional
    for (int64_t k0 = 0; k0 < cols; k0 += 8 * 256) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int64_t k = k0 + threadIdx.x + 256 * u;
        v[u] = fabsf(xr[k < cols ? k : cols - 1]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (v[u] < __builtin_huge_valf() && v[u] > mx) mx = v[u];
    }
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  if (threadIdx.x == 0) atomicMax(amax, __float_as_uint(red[0]));
}

// dst[0][r][k] = hi, dst[1][r][k] = lo of X[r][k] * 2^(14 - ilogb(amax)), zero for k >= cols
__global__ __launch_bounds__(256) void split_kernel(const float* __restrict__ X, int64_t rows, int64_t cols,
                                                    int64_t ld, const unsigned* __restrict__ amax,
                                                    _Float16* __restrict__ dst, int64_t k64) {
  const int64_t r = blockIdx.y;
  const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (k >= k64) return;
  const float mx = __uint_as_float(amax[0]);
  const float sc = (mx > 0.f) ? ldexpf(1.f, 14 - ilogbf(mx)) : 1.f;
  _Float16 hi = (_Float16)0, lo = (_Float16)0;
  if (k < cols) {
    const float v = X[r * ld + k] * sc;
    hi = (_Float16)v;
    lo = (_Float16)(v - (float)hi);
  }
  dst[r * k64 + k] = hi;
  dst[(rows + r) * k64 + k] = lo;
}

// C = (sum over the three piece pairs of A_p B_p^T) / (scale_A scale_B)
__global__ __launch_bounds__(64 * GNW) void gemm_split_kernel(const _Float16* __restrict__ As,
                                                              const _Float16* __restrict__ Bs, int64_t M,
                                                              int64_t N, int64_t k64,
                                                              const unsigned* __restrict__ amaxA,
                                                              const unsigned* __restrict__ amaxB,
                                                              float* __restrict__ C, int64_t ldc) {
  // Workgroups are dealt to the 8 XCDs round-robin by flat index; each XCD takes a
  // contiguous run of the row-major tile list, so that its workgroups share rows of A.
  const int tm = (int)ceil_div(M, GT), tn = (int)ceil_div(N, GT);
  const int64_t total = (int64_t)tm * tn;
  const int64_t per = (total + 7) / 8;
  const int64_t q = blockIdx.x >> 3;
  const int64_t item = (int64_t)(blockIdx.x & 7) * per + q;
  if (q >= per || item >= total) return;
  const int bm = (int)(item / tn), bn = (int)(item % tn);

  extern __shared__ __attribute__((aligned(16))) unsigned char gsm[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)gsm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 2, wc = wave & 3;
  const int kh = lane >> 5, l32 = lane & 31;
  const int64_t m0 = (int64_t)bm * GT, n0 = (int64_t)bn * GT;
  const int64_t rowsA = (M - m0 < GT) ? M - m0 : GT, rowsB = (N - n0 < GT) ? N - n0 : GT;

  const int dr = lane >> 3;
  const int dc = (lane & 7) ^ dr;
  uint32_t voff[GDPW];
#pragma unroll
  for (int j = 0; j < GDPW; ++j)
    voff[j] = (uint32_t)(((int64_t)((wave + GNW * j) * 8 + dr) * k64 + dc * 8) * 2);

  const int nk1 = (int)(k64 / GK);          // steps per piece pair
  const int nk = 3 * nk1;
  int4v rsA, rsB;
  auto set_piece = [&](int p) {
    // piece pairs (A, B): (hi, hi), (hi, lo), (lo, hi)
    const int64_t pa = (p == 2) ? M : 0, pb = (p == 1) ? N : 0;
    rsA = make_rsrc(As + (pa + m0) * k64, rowsA * k64 * 2);
    rsB = make_rsrc(Bs + (pb + n0) * k64, rowsB * k64 * 2);
  };
  auto issue = [&](int s, int st) {
    const uint32_t soff = (uint32_t)((s % nk1) * GK * 2);
    const uint32_t sbase = lds0 + st * GSTAGEB;
#pragma unroll
    for (int j = 0; j < GDPW; ++j) {
      load16_to_lds(rsA, sbase + (wave + GNW * j) * 1024, voff[j], soff);
      load16_to_lds(rsB, sbase + GTILEB + (wave + GNW * j) * 1024, voff[j], soff);
    }
  };

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int rswz = l32 & 7;
  set_piece(0);
  issue(0, 0);
  int st = 0;
#pragma unroll 1
  for (int s = 0; s < nk; ++s) {
    wait_all_loads();
    __syncthreads();
    if (s + 1 < nk) {
      if ((s + 1) % nk1 == 0) set_piece((s + 1) / nk1);
      issue(s + 1, st ^ 1);
    }
    const unsigned char* Asm = gsm + st * GSTAGEB;
    const unsigned char* Bsm = Asm + GTILEB;
#pragma unroll
    for (int ks = 0; ks < GK / 16; ++ks) {
      half8 af[4], bfr[2];
      const int cpos = ((2 * ks + kh) ^ rswz) * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        af[i] = *reinterpret_cast<const half8*>(Asm + (wr * 128 + i * 32 + l32) * GROWB + cpos);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        bfr[j] = *reinterpret_cast<const half8*>(Bsm + (wc * 64 + j * 32 + l32) * GROWB + cpos);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    st ^= 1;
  }

  const float ma = __uint_as_float(amaxA[0]), mb = __uint_as_float(amaxB[0]);
  const int ea = (ma > 0.f) ? 14 - ilogbf(ma) : 0, eb = (mb > 0.f) ? 14 - ilogbf(mb) : 0;
  const float inv = ldexpf(1.f, -ea) * ldexpf(1.f, -eb);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t col = n0 + wc * 64 + j * 32 + l32;
      if (col >= N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wr * 128 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
        if (row < M) C[row * ldc + col] = acc[i][j][v] * inv;
      }
    }
}

inline int64_t k64_of(int64_t K) { return ceil_div(K, GK) * GK; }

}  // namespace

size_t gemm_split_scratch_bytes(int64_t M, int64_t N, int64_t K) {
  const int64_t k64 = k64_of(K);
  return kAlign + align_up((size_t)2 * M * k64 * sizeof(_Float16)) + align_up((size_t)2 * N * k64 * sizeof(_Float16));
}

// C (M x N) = A (M x K) * B (N x K)^T.  scratch: [amaxA, amaxB][A pieces][B pieces].
// b_ready != 0: the pieces of B in scratch are those of an earlier call with the same B.
hipError_t launch_gemm_split(hipStream_t s, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
                             const float* B, int64_t ldb, float* C, int64_t ldc, void* scratch, int b_ready) {
  const int64_t k64 = k64_of(K);
  unsigned* amax = (unsigned*)scratch;
  _Float16* As = (_Float16*)((char*)scratch + kAlign);
  _Float16* Bs = (_Float16*)((char*)As + align_up((size_t)2 * M * k64 * sizeof(_Float16)));
  hipError_t e;
  static std::atomic<uint64_t> lds_set{0};
  if ((e = ensure_dynamic_lds((const void*)gemm_split_kernel, 2 * GSTAGEB, lds_set)) != hipSuccess) return e;
  // amax words are cleared by a small kernel (capturable, unlike a memset node)
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, amax, b_ready ? 1 : 2, 0u);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)(M < 2048 ? M : 2048)), dim3(256), 0, s, A, M, K, lda, amax);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(split_kernel, dim3((unsigned)ceil_div(k64, 256), (unsigned)M), dim3(256), 0, s, A, M, K, lda,
                     amax, As, k64);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (!b_ready) {
    hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)(N < 2048 ? N : 2048)), dim3(256), 0, s, B, N, K, ldb, amax + 1);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(split_kernel, dim3((unsigned)ceil_div(k64, 256), (unsigned)N), dim3(256), 0, s, B, N, K,
                       ldb, amax + 1, Bs, k64);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const int64_t total = ceil_div(M, GT) * ceil_div(N, GT);
  hipLaunchKernelGGL(gemm_split_kernel, dim3((unsigned)(8 * ceil_div(total, 8))), dim3(64 * GNW), 2 * GSTAGEB, s,
                     As, Bs, M, N, k64, amax, amax + 1, C, ldc);
  return hipGetLastError();
}

}  // namespace ganq
