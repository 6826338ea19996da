// H = X X^T (Algorithm 1; Eq. (9)) for fp16 activations on the gfx950 matrix
// cores: fp16 x fp16 products, fp32 accumulation (v_mfma_f32_32x32x16_f16).
//
// X is n x p row-major, so both operands of the product are k-contiguous.
// Only the 256 x 256 tiles on or below the diagonal are computed (H is symmetric); the
// token axis is split across workgroups so that small n still fills the chip,
// each split writes its partial tile to scratch, and a second kernel sums the
// partials in a fixed order (bit-reproducible, no float atomics) and writes
// both triangles of H.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int HT = kHessTile;   // 256 x 256 output tile per workgroup
constexpr int HK = 32;          // k per LDS stage
constexpr int HPAD = 8;         // halfs of row padding in LDS
constexpr int HLD = HK + HPAD;
constexpr int HSTAGE = 2 * HT * HLD * 2;   // bytes of one stage: A tile + B tile

// Eight consecutive halfs of row `row` from column k, zero outside [0, n) x [., kend).
__device__ inline half8 load_half8(const _Float16* __restrict__ X, int64_t row, int64_t k,
                                   int64_t n, int64_t kend, int64_t ldx) {
  half8 r;
  if (row < n && k + 7 < kend) {
    r = *reinterpret_cast<const half8*>(X + row * ldx + k);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (row < n && k + i < kend) ? X[row * ldx + k + i] : (_Float16)0;
  }
  return r;
}

// 4 wavefronts in a 2 x 2 grid, each owning a 128 x 128 sub-tile as 4 x 4 MFMA tiles of
// 32 x 32 (256 accumulator registers): 16 MFMAs per 8 LDS fragment reads keeps the LDS at
// half of its bandwidth.  Two LDS stages, one barrier per k-step: while a stage is being
// multiplied the registers fetched one step earlier are written to the other stage and the
// loads of the step after that are issued.
__device__ inline void hessian_tile(const _Float16* __restrict__ X, int64_t n, int64_t p, int64_t ldx,
                                    int64_t chunk, float* __restrict__ partials) {
  // triangular tile index -> (bm, bn), bn <= bm
  const int t = blockIdx.x;
  int bm = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
  while ((int64_t)(bm + 1) * (bm + 2) / 2 <= t) ++bm;
  while ((int64_t)bm * (bm + 1) / 2 > t) --bm;
  const int bn = t - (int)((int64_t)bm * (bm + 1) / 2);
  const int split = blockIdx.y;
  const int64_t kbeg = (int64_t)split * chunk;
  const int64_t kend = (kbeg + chunk < p) ? kbeg + chunk : p;

  extern __shared__ __attribute__((aligned(16))) unsigned char hsm[];
  auto As_of = [&](int st) { return reinterpret_cast<_Float16 (*)[HLD]>(hsm + st * HSTAGE); };
  auto Bs_of = [&](int st) { return reinterpret_cast<_Float16 (*)[HLD]>(hsm + st * HSTAGE + HT * HLD * 2); };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int kh = lane >> 5, l32 = lane & 31;
  const int64_t m0 = (int64_t)bm * HT, n0 = (int64_t)bn * HT;

  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int lrow = tid >> 2, lk = (tid & 3) * 8;
  half8 ra[4], rb[4];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      ra[ps] = load_half8(X, m0 + lrow + 64 * ps, k0 + lk, n, kend, ldx);
      rb[ps] = load_half8(X, n0 + lrow + 64 * ps, k0 + lk, n, kend, ldx);
    }
  };
  auto stage_regs = [&](int st) {
    _Float16 (*As)[HLD] = As_of(st);
    _Float16 (*Bs)[HLD] = Bs_of(st);
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      *reinterpret_cast<half8*>(&As[lrow + 64 * ps][lk]) = ra[ps];
      *reinterpret_cast<half8*>(&Bs[lrow + 64 * ps][lk]) = rb[ps];
    }
  };

  if (kbeg < kend) {
    fetch(kbeg);
    stage_regs(0);
    if (kbeg + HK < kend) fetch(kbeg + HK);
  }
  int st = 0;
#pragma unroll 1
  for (int64_t k0 = kbeg; k0 < kend; k0 += HK) {
    __syncthreads();
    _Float16 (*As)[HLD] = As_of(st);
    _Float16 (*Bs)[HLD] = Bs_of(st);
#pragma unroll
    for (int ks = 0; ks < HK; ks += 16) {
      half8 af[4], bfr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        af[i] = *reinterpret_cast<const half8*>(&As[wr * 128 + i * 32 + l32][ks + 8 * kh]);
        bfr[i] = *reinterpret_cast<const half8*>(&Bs[wc * 128 + i * 32 + l32][ks + 8 * kh]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (k0 + HK < kend) {
      stage_regs(st ^ 1);
      if (k0 + 2 * HK < kend) fetch(k0 + 2 * HK);
    }
    st ^= 1;
  }

  float* out = partials + (int64_t)split * n * n;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = n0 + wc * 128 + j * 32 + l32;
      if (col >= n) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wr * 128 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
        if (row < n && col <= row) out[row * n + col] = acc[i][j][v];
      }
    }
}

__global__ __launch_bounds__(256) void hessian_f16_kernel(const _Float16* __restrict__ X, int64_t n,
                                                          int64_t p, int64_t ldx, int64_t chunk,
                                                          float* __restrict__ partials) {
  hessian_tile(X, n, p, ldx, chunk, partials);
}

// H[i][j] = H[j][i] = (accumulate ? H[i][j] : 0) + sum_s src[s][i][j] for i >= j.
__global__ __launch_bounds__(256) void reduce_mirror_kernel(float* __restrict__ H, int64_t n,
                                                            int64_t ldh,
                                                            const float* __restrict__ src,
                                                            int64_t lds, int nsplit,
                                                            int accumulate) {
  const int bi = blockIdx.y, bj = blockIdx.x;
  if (bj > bi) return;
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int64_t i = (int64_t)bi * 32 + r, j = (int64_t)bj * 32 + tx;
    float v = 0.f;
    if (i < n && j < n && j <= i) {
      for (int s = 0; s < nsplit; ++s) v += src[(int64_t)s * lds * n + i * lds + j];
      if (accumulate) v += H[i * ldh + j];
      H[i * ldh + j] = v;
    }
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    // element (i, j) of the tile goes to H[j][i]; write rows of the transposed tile
    const int64_t jj = (int64_t)bj * 32 + r, ii = (int64_t)bi * 32 + tx;
    if (ii < n && jj < n && jj < ii) H[jj * ldh + ii] = tile[tx][r];
  }
}

}  // namespace

int hessian_split(int64_t n, int64_t p) {
  const int64_t nt = ceil_div(n, HT);
  const int64_t tiles = nt * (nt + 1) / 2;
  int split = 1;
  while (split < kHessMaxSplit && tiles * split < 1024 && p / (split * 2) >= 2048) split *= 2;
  return split;
}

size_t hessian_scratch_bytes(int64_t n, int64_t p) {
  if (p <= 0) return 0;
  return align_up((size_t)hessian_split(n, p) * (size_t)n * (size_t)n * sizeof(float));
}

hipError_t launch_hessian_f16(hipStream_t s, const _Float16* X, int64_t n, int64_t p, int64_t ldx,
                              float* H, int64_t ldh, int accumulate, float* partials) {
  const int split = hessian_split(n, p);
  int64_t chunk = ceil_div(ceil_div(p, split), HK) * HK;
  const int64_t nt = ceil_div(n, HT);
  dim3 grid((unsigned)(nt * (nt + 1) / 2), (unsigned)split);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t ea = hipFuncSetAttribute((const void*)hessian_f16_kernel,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 2 * HSTAGE);
    if (ea != hipSuccess) return ea;
    attr_set = true;
  }
  hipLaunchKernelGGL(hessian_f16_kernel, grid, dim3(256), 2 * HSTAGE, s, X, n, p, ldx, chunk, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  hipLaunchKernelGGL(reduce_mirror_kernel, g2, dim3(256), 0, s, H, n, ldh, partials, n, split,
                     accumulate);
  return hipGetLastError();
}

hipError_t launch_mirror_lower(hipStream_t s, float* H, int64_t n, int64_t ldh, const float* src,
                               int64_t lds, int accumulate) {
  dim3 g2((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  hipLaunchKernelGGL(reduce_mirror_kernel, g2, dim3(256), 0, s, H, n, ldh, src, lds, 1, accumulate);
  return hipGetLastError();
}

}  // namespace ganq
