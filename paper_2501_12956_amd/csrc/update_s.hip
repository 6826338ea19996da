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
//            on the matrix cores (v_mfma_f32_16x16x4_f32).  The later columns
//            are split over the 4 wavefronts; each wavefront streams its share
//            of L straight from L2 into registers, software-pipelined 8 MFMA
//            groups deep, and the 4 partial tiles are summed through LDS in a
//            fixed order.  This is the sum of Eq. (22) restricted to columns
//            right of the block, re-associated.
//   phase 2  the 64 columns of the block one by one, 16 lanes per row.  Each
//            row's codebook is sorted once (stable); lane c holds the midpoint
//            between sorted codes c and c+1, so the nearest code of a target
//            is the number of midpoints below it: one compare, one ballot, one
//            popcount.  The residual of the chosen code is picked out of the 16
//            lanes with an exact one-hot lane-row sum (DPP), and the block's
//            remaining accumulators get a rank-1 update with the row of L held
//            in LDS.  A target exactly on a midpoint takes the lower code; two
//            equal codes resolve to the lower index.
// The slab's residuals E live in scratch in a (column, row-in-slab) layout so
// that one MFMA operand fetch is 64 consecutive floats.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int SB = 64;          // columns per block
constexpr int SR = kSlabRows;   // rows per workgroup
constexpr int PU = 8;           // MFMA groups per software-pipeline stage

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
template <int K>
__device__ inline int row_bcast_i(int v) { return dpp_i<0x150 + K>(v); }

// sum over the 16 lanes of a row; every lane gets the result
__device__ inline float row_sum_f(float d) {
  d += dpp_f<0xB1>(d);    // quad_perm [1,0,3,2]
  d += dpp_f<0x4E>(d);    // quad_perm [2,3,0,1]
  d += dpp_f<0x141>(d);   // row_half_mirror
  d += dpp_f<0x140>(d);   // row_mirror
  return d;
}

// Stable rank of this lane's code within its row, and "is lane k's code equal to mine".
template <int K>
struct RankLoop {
  __device__ static inline void run(float tc, int c, int& rank) {
    const float tk = row_bcast<K>(tc);
    rank += (tk < tc || (tk == tc && K < c)) ? 1 : 0;
    if constexpr (K > 0) RankLoop<K - 1>::run(tc, c, rank);
  }
};
template <int K>
struct RepLoop {
  // lowest original index among the sorted positions that hold the same value as mine
  __device__ static inline void run(float ts, int orig, int& rep) {
    const float tk = row_bcast<K>(ts);
    const int ok = row_bcast_i<K>(orig);
    if (tk == ts && ok < rep) rep = ok;
    if constexpr (K > 0) RepLoop<K - 1>::run(ts, orig, rep);
  }
};

template <int JL>
struct Step {
  // One column of phase 2 (local column JL of the block).
  __device__ static inline void run(int bw, int c, int gshift, float ts, float mid,
                                    const float (&Wr)[4], const float (&rd)[4], float (&acc)[4],
                                    float (&Er)[4], int (&Ir)[4], const float (*Ld)[SB + 4]) {
    if (JL < bw) {
      constexpr int co = JL & 15, qo = JL >> 4;
      const float tg = row_bcast<co>(fmaf(acc[qo], rd[qo], Wr[qo]));
      const unsigned long long vote = __builtin_amdgcn_ballot_w64(tg > mid);
      const int idx = __builtin_popcount((unsigned)(vote >> gshift) & 0xffffu);
      const float cand = row_bcast<co>(Wr[qo]) - ts;
      const float e = row_sum_f((c == idx) ? cand : 0.f);
      if (c == co) {
        Er[qo] = e;
        Ir[qo] = idx;
      }
#pragma unroll
      for (int q = 0; q <= qo; ++q) acc[q] = fmaf(e, Ld[JL][16 * q + c], acc[q]);
    }
    if constexpr (JL > 0) Step<JL - 1>::run(bw, c, gshift, ts, mid, Wr, rd, acc, Er, Ir, Ld);
  }
};

__global__ __launch_bounds__(256) void rdiag_kernel(const float* __restrict__ L, int64_t n,
                                                    int64_t ldl, float* __restrict__ rdiag) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < n) rdiag[j] = 1.f / L[j * ldl + j];
}

struct LFrag {
  float a;
  float4 b;
};

__global__ __launch_bounds__(256) void update_S_kernel(const float* __restrict__ W, int64_t m,
                                                       int64_t n, int64_t ldw,
                                                       const float* __restrict__ L, int64_t ldl,
                                                       const float* __restrict__ rdiag,
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

  // ---- sort this row's codebook (stable), build midpoints and tie representatives ----
  float tc = __builtin_huge_valf();
  if (c < C) tc = row_ok ? T[row * C + c] : 0.f;
  int rank = 0;
  RankLoop<15>::run(tc, c, rank);
  const int paddr = ((lane & 48) | rank) << 2;
  const float ts = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(paddr, __builtin_bit_cast(int, tc)));
  const int orig = __builtin_amdgcn_ds_permute(paddr, c);
  int rep = orig;
  RepLoop<15>::run(ts, orig, rep);
  const float tnext = dpp_f<0x101>(ts);             // row_shl:1 -> value of lane c + 1
  const float mid = (c < 15) ? 0.5f * (ts + tnext) : __builtin_huge_valf();
  const int gshift = 16 * g;

  const int nblk = (int)ceil_div(n, SB);
  for (int b = nblk - 1; b >= 0; --b) {
    const int64_t j0 = (int64_t)b * SB;
    const int bw = (int)((n - j0 < SB) ? n - j0 : SB);
    const int64_t kstart = j0 + SB;

    // ---- stage the diagonal block of L and this block's W ----
    for (int e4 = tid; e4 < SB * SB / 4; e4 += 256) {
      const int rr = e4 / (SB / 4), cc = (e4 % (SB / 4)) * 4;
      const int64_t gr = j0 + rr, gc = j0 + cc;
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if (gr < n && cc < rr) {
        if (vecL && gc + 3 < n) {
          const float4 q4 = *reinterpret_cast<const float4*>(L + gr * ldl + gc);
          v[0] = q4.x; v[1] = q4.y; v[2] = q4.z; v[3] = q4.w;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (gc + i < n) ? L[gr * ldl + gc + i] : 0.f;
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) Ld[rr][cc + i] = (cc + i < rr) ? v[i] : 0.f;
    }
    float Wr[4], rd[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t col = j0 + 16 * q + c;
      Wr[q] = (row_ok && col < n) ? W[row * ldw + col] : 0.f;
      rd[q] = (col < n) ? rdiag[col] : 0.f;
    }

    // ---- phase 1: acc = E[:, kstart:] * L[kstart:, block] on the matrix cores ----
    floatx4 macc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) macc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (kstart < n) {
      const float* __restrict__ Lcol = L + j0 + 4 * c;
      const float* __restrict__ Ecol = Eslab + c;
      auto fetch = [&](int64_t k) {
        LFrag f;
        f.a = Ecol[k * SR];
        if (vecL) {
          f.b = *reinterpret_cast<const float4*>(Lcol + k * ldl);
        } else {
          f.b.x = Lcol[k * ldl]; f.b.y = Lcol[k * ldl + 1];
          f.b.z = Lcol[k * ldl + 2]; f.b.w = Lcol[k * ldl + 3];
        }
        return f;
      };
      auto mma = [&](const LFrag& f) {
        macc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a, f.b.x, macc[0], 0, 0, 0);
        macc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a, f.b.y, macc[1], 0, 0, 0);
        macc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a, f.b.z, macc[2], 0, 0, 0);
        macc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a, f.b.w, macc[3], 0, 0, 0);
      };
      // this wavefront takes the k-quads qd = wave, wave + 4, ...; lane row g adds to k
      const int64_t nfull = (n - kstart) / 4;                 // quads with all 4 rows < n
      const int64_t myfull = (nfull > wave) ? (nfull - wave + 3) / 4 : 0;
      const int64_t kbase = kstart + 4 * wave + g;            // k of iteration 0
      int64_t it = 0;
      if (myfull >= PU) {
        LFrag cur[PU], nxt[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) cur[u] = fetch(kbase + 16 * (it + u));
        it += PU;
        for (; it + PU <= myfull; it += PU) {
#pragma unroll
          for (int u = 0; u < PU; ++u) nxt[u] = fetch(kbase + 16 * (it + u));
#pragma unroll
          for (int u = 0; u < PU; ++u) mma(cur[u]);
#pragma unroll
          for (int u = 0; u < PU; ++u) cur[u] = nxt[u];
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) mma(cur[u]);
      }
      for (; it < myfull; ++it) mma(fetch(kbase + 16 * it));
      // ragged last quad (n - kstart not a multiple of 4): one wavefront, rows masked
      if ((n - kstart) % 4 != 0 && (nfull % 4) == wave) {
        const int64_t k = kstart + 4 * nfull + g;
        LFrag f;
        f.a = 0.f;
        f.b = float4{0.f, 0.f, 0.f, 0.f};
        if (k < n) f = fetch(k);
        mma(f);
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
    int Ir[4] = {0, 0, 0, 0};
    Step<SB - 1>::run(bw, c, gshift, ts, mid, Wr, rd, acc, Er, Ir, Ld);

#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t col = j0 + 16 * q + c;
      const int qi = __shfl(rep, (lane & 48) | Ir[q], 64);     // sorted position -> original index
      if (col < n) {
        Eslab[col * SR + r] = Er[q];
        if (row_ok) {
          Q[row * ldq + col] = (uint8_t)qi;
          if (E != nullptr) E[row * lde + col] = Er[q];
        }
      }
    }
    __syncthreads();   // E of this block visible to all wavefronts; LDS reusable
  }
}

}  // namespace

size_t update_s_scratch_bytes(int64_t m, int64_t n) {
  return align_up((size_t)pad_rows(m) * (size_t)n * sizeof(float)) + align_up((size_t)n * sizeof(float));
}

hipError_t launch_update_S(hipStream_t s, const float* W, int64_t m, int64_t n, int64_t ldw,
                           const float* L, int64_t ldl, const float* T, int nbits, uint8_t* Q,
                           int64_t ldq, float* E, int64_t lde, void* scratch) {
  const int vecL = (ldl % 4 == 0) && (((uintptr_t)L) % 16 == 0);
  float* Es = (float*)scratch;
  float* rdiag = (float*)((char*)scratch + align_up((size_t)pad_rows(m) * (size_t)n * sizeof(float)));
  hipLaunchKernelGGL(rdiag_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, L, n, ldl, rdiag);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(update_S_kernel, dim3((unsigned)ceil_div(m, SR)), dim3(256), 0, s, W, m, n,
                     ldw, L, ldl, rdiag, T, 1 << nbits, Q, ldq, E, lde, Es, vecL);
  return hipGetLastError();
}

}  // namespace ganq
