// S-update of GANQ: back-substitution on the Cholesky factor L, Eq. (13)-(22)
// and the inner loop of Algorithm 1.
//
// For j = n-1 .. 0 and every row i:
//     tgt  = W_ij + (sum_{u>j} E_iu L_uj) / L_jj,     E_iu = W_iu - T_i[Q_iu]
//     Q_ij = argmin_s |tgt - T_is|   (lowest s on ties)
//
// Rows are independent and columns are sequential, so one workgroup owns a
// slab of 16 rows and walks all n columns by itself - no grid-wide
// synchronisation.  Columns are taken in blocks of 64 from the right:
//   phase 1  acc[16 x 64] = E[16 x later columns] * L[later rows, block]
//            on the matrix cores (v_mfma_f32_16x16x4_f32), the later columns
//            split over the 4 wavefronts and reduced through LDS in a fixed
//            order; this is the sum of Eq. (22) restricted to columns right of
//            the block, re-associated;
//   phase 2  the 64 columns of the block one by one: 16 lanes per row, one
//            lane per code; lane-row broadcasts (DPP) of the target, a 16-lane
//            min-reduction of the distance and of the lowest index attaining
//            it, then a rank-1 update of the block's remaining accumulators
//            with the row of L held in LDS.
// The slab's residuals E live in scratch in a (column, row-in-slab) layout so
// that one MFMA operand fetch is 64 consecutive floats.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int SB = 64;          // columns per block
constexpr int SR = kSlabRows;   // rows per workgroup

template <int CTRL>
__device__ inline float dpp_f(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ inline int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
// value of lane K of this lane's 16-lane row
template <int K>
__device__ inline float row_bcast(float v) { return dpp_f<0x150 + K>(v); }

// min over the 16 lanes of a row; every lane gets the result
__device__ inline float row_min_f(float d) {
  d = fminf(d, dpp_f<0xB1>(d));    // quad_perm [1,0,3,2]
  d = fminf(d, dpp_f<0x4E>(d));    // quad_perm [2,3,0,1]
  d = fminf(d, dpp_f<0x141>(d));   // row_half_mirror
  d = fminf(d, dpp_f<0x140>(d));   // row_mirror
  return d;
}
__device__ inline int row_min_i(int d) {
  d = min(d, dpp_i<0xB1>(d));
  d = min(d, dpp_i<0x4E>(d));
  d = min(d, dpp_i<0x141>(d));
  d = min(d, dpp_i<0x140>(d));
  return d;
}

template <int JL>
struct Step {
  // One column of phase 2 (local column JL of the block).
  __device__ static inline void run(int bw, int c, int lane, int C, float tc, const float (&Wr)[4],
                                    const float (&rd)[4], float (&acc)[4], float (&Er)[4],
                                    int (&Qr)[4], const float (*Ld)[SB + 4]) {
    if (JL < bw) {
      constexpr int co = JL & 15, qo = JL >> 4;
      const float tg = row_bcast<co>(fmaf(acc[qo], rd[qo], Wr[qo]));
      const float d = fabsf(tg - tc);
      const float dmin = row_min_f(d);
      int idx = row_min_i((d == dmin) ? c : 16);
      idx = min(idx, C - 1);
      const float tsel = __shfl(tc, (lane & 48) | idx, 64);
      const float e = row_bcast<co>(Wr[qo]) - tsel;
      if (c == co) {
        Er[qo] = e;
        Qr[qo] = idx;
      }
#pragma unroll
      for (int q = 0; q <= qo; ++q) acc[q] = fmaf(e, Ld[JL][16 * q + c], acc[q]);
    }
    if constexpr (JL > 0) Step<JL - 1>::run(bw, c, lane, C, tc, Wr, rd, acc, Er, Qr, Ld);
  }
};

__global__ __launch_bounds__(256) void update_S_kernel(const float* __restrict__ W, int64_t m,
                                                       int64_t n, int64_t ldw,
                                                       const float* __restrict__ L, int64_t ldl,
                                                       const float* __restrict__ T, int C,
                                                       uint8_t* __restrict__ Q, int64_t ldq,
                                                       float* __restrict__ E, int64_t lde,
                                                       float* __restrict__ Es, int vecL) {
  __shared__ float Ld[SB][SB + 4];        // diagonal block of L (row = later column)
  __shared__ float red[4][4][4][64];      // [wave][t][v][lane] partial accumulators

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int r = 4 * wave + g;                       // row within the slab (phase 2)
  const int64_t row0 = (int64_t)blockIdx.x * SR;
  const int64_t row = row0 + r;
  const bool row_ok = row < m;
  float* __restrict__ Eslab = Es + (int64_t)blockIdx.x * n * SR;

  float tc = __builtin_huge_valf();
  if (c < C) tc = row_ok ? T[row * C + c] : 0.f;

  const int nblk = (int)ceil_div(n, SB);
  for (int b = nblk - 1; b >= 0; --b) {
    const int64_t j0 = (int64_t)b * SB;
    const int bw = (int)((n - j0 < SB) ? n - j0 : SB);
    const int64_t kstart = j0 + SB;

    // ---- stage the diagonal block of L and this block's W ----
    for (int e4 = tid; e4 < SB * SB / 4; e4 += 256) {
      const int rr = e4 / (SB / 4), cc = (e4 % (SB / 4)) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int64_t gr = j0 + rr, gc = j0 + cc + i;
        Ld[rr][cc + i] = (gr < n && gc < n && gc < gr) ? L[gr * ldl + gc] : 0.f;
      }
    }
    float Wr[4], rd[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t col = j0 + 16 * q + c;
      Wr[q] = (row_ok && col < n) ? W[row * ldw + col] : 0.f;
      rd[q] = (col < n) ? 1.f / L[col * ldl + col] : 0.f;
    }

    // ---- phase 1: acc = E[:, kstart:] * L[kstart:, block] on the matrix cores ----
    floatx4 macc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) macc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (kstart < n) {
      const int64_t nquad = ceil_div(n - kstart, 4);
      const float* __restrict__ Lcol = L + j0 + 4 * c;
#pragma unroll 4
      for (int64_t qd = wave; qd < nquad; qd += 4) {
        const int64_t k = kstart + 4 * qd + g;
        float a = 0.f;
        float bv[4] = {0.f, 0.f, 0.f, 0.f};
        if (k < n) {
          a = Eslab[k * SR + c];
          if (vecL) {
            const float4 q4 = *reinterpret_cast<const float4*>(Lcol + k * ldl);
            bv[0] = q4.x; bv[1] = q4.y; bv[2] = q4.z; bv[3] = q4.w;
          } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) bv[t] = Lcol[k * ldl + t];
          }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
          macc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv[t], macc[t], 0, 0, 0);
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][t][v][lane] = macc[t][v];
    __syncthreads();

    // MFMA tile t, lane l', register v holds (row 4*(l'/16) + v, local column 4*(l'%16) + t)
    float acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int jl = 16 * q + c;
      const int sl = 16 * wave + (jl >> 2), t = jl & 3;
      acc[q] = (red[0][t][g][sl] + red[1][t][g][sl]) + (red[2][t][g][sl] + red[3][t][g][sl]);
    }

    // ---- phase 2: the block's columns, right to left ----
    float Er[4] = {0.f, 0.f, 0.f, 0.f};
    int Qr[4] = {0, 0, 0, 0};
    Step<SB - 1>::run(bw, c, lane, C, tc, Wr, rd, acc, Er, Qr, Ld);

#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t col = j0 + 16 * q + c;
      if (col < n) {
        Eslab[col * SR + r] = Er[q];
        if (row_ok) {
          Q[row * ldq + col] = (uint8_t)Qr[q];
          if (E != nullptr) E[row * lde + col] = Er[q];
        }
      }
    }
    __syncthreads();   // E of this block visible to all wavefronts; LDS reusable
  }
}

}  // namespace

size_t update_s_scratch_bytes(int64_t m, int64_t n) {
  return align_up((size_t)pad_rows(m) * (size_t)n * sizeof(float));
}

hipError_t launch_update_S(hipStream_t s, const float* W, int64_t m, int64_t n, int64_t ldw,
                           const float* L, int64_t ldl, const float* T, int nbits, uint8_t* Q,
                           int64_t ldq, float* E, int64_t lde, void* scratch) {
  const int vecL = (ldl % 4 == 0) && (((uintptr_t)L) % 16 == 0);
  hipLaunchKernelGGL(update_S_kernel, dim3((unsigned)ceil_div(m, SR)), dim3(256), 0, s, W, m, n,
                     ldw, L, ldl, T, 1 << nbits, Q, ldq, E, lde, (float*)scratch, vecL);
  return hipGetLastError();
}

}  // namespace ganq
