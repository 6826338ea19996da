// L = Cholesky(H) or of its preconditioned form (Eq. (10), Remark 3.1,
// Appendix A Eq. (23)-(24)), blocked, fp32 storage.
//
// The lower triangle of H (plus the preconditioner) is copied to a working matrix W; L is
// written once and never read back as input of the same kernel that writes it.  Columns go
// in outer panels of 256, each of four inner blocks of 64:
//   inner block (one launch): every workgroup owns 64 rows below the diagonal block and
//     repeats the small shared part itself - it brings the 64 x 64 diagonal block up to date
//     with the earlier inner blocks of the panel (left-looking, from L), factors it and
//     inverts the factor in LDS - then updates its own rows the same way and multiplies
//     them by that inverse.  No second launch and no grid-wide dependency for the solve.
//   outer panel: W22 -= L21 L21^T with K = 256 on the fp32 matrix-core GEMM.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int NB = 64;

__global__ void fill_i32_kernel(int* p, int v) { *p = v; }

// W <- lower triangle of H (+ preconditioner on the diagonal), L <- 0.
// delta (if used) must already hold the diagonal offsets.
// thr[i] = pivot threshold of column i: tau times the diagonal entry that is factorised.
// One thread takes four consecutive columns (16-byte loads and stores where VEC says that rows of
// H, W and L allow them).  Entries of W right of the diagonal inside the group that holds the
// diagonal are written as 0; the rest of the upper triangle of W is never read.
template <bool VEC>
__global__ __launch_bounds__(256) void copy_lower_kernel(const float* __restrict__ H, int64_t n,
                                                         int64_t ldh, float* __restrict__ W,
                                                         float* __restrict__ L, int64_t ldl,
                                                         int precond, float lambda,
                                                         const float* __restrict__ delta, float tau,
                                                         float* __restrict__ thr) {
  const int64_t j0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const int64_t i = blockIdx.y;
  if (j0 >= n) return;
  const int cnt = (int)((n - j0 < 4) ? n - j0 : 4);
  if (VEC) {
    *reinterpret_cast<float4*>(L + i * ldl + j0) = float4{0.f, 0.f, 0.f, 0.f};
  } else {
    for (int t = 0; t < cnt; ++t) L[i * ldl + j0 + t] = 0.f;
  }
  if (j0 > i) return;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  if (VEC) {
    const float4 h = *reinterpret_cast<const float4*>(H + i * ldh + j0);
    v[0] = h.x; v[1] = h.y; v[2] = h.z; v[3] = h.w;
  } else {
    for (int t = 0; t < cnt; ++t) v[t] = H[i * ldh + j0 + t];
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int64_t j = j0 + t;
    if (j > i) v[t] = 0.f;
    if (j == i) {
      if (precond == GANQ_PRECOND_LAMBDA) v[t] += lambda;
      if (precond == GANQ_PRECOND_DIAGDOM) v[t] += delta[i];
      // a diagonal that is not positive and finite fails at once (threshold +inf: no pivot passes)
      thr[i] = (v[t] > 0.f && v[t] < 3.0e38f) ? tau * v[t] : __builtin_huge_valf();
    }
  }
  if (VEC) {
    *reinterpret_cast<float4*>(W + i * n + j0) = float4{v[0], v[1], v[2], v[3]};
  } else {
    for (int t = 0; t < cnt; ++t)
      if (j0 + t <= i) W[i * n + j0 + t] = v[t];
  }
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

// ---- 64 x 64 diagonal block: factor and inverse of the factor, one workgroup ----
//
// The block lives in LDS and is processed as 4 x 4 leaves of 16 x 16.  Per leaf column kb:
// (a) one wavefront factors the 16 x 16 diagonal leaf with its rows in lanes 0..15 and its
//     columns in registers - pivots and multipliers travel by v_readlane, no LDS round trip
//     and no barrier inside the 16 steps - and inverts the leaf factor by forward
//     substitution (one column per lane);
// (b) all threads form the leaf panel below it, P = A21 * inv(L11)^T;
// (c) all threads apply  A22 -= P P^T  to the rest of the block.
// The inverse of the whole 64 x 64 factor is then assembled from the leaf inverses by block
// forward substitution, one block diagonal per level.  Three barriers per leaf column and two
// per level instead of one per matrix column.  On a bad pivot the 1-based global index of
// the first one is recorded in *info (if still 0) and the pivot is replaced by 1 so that
// the kernel terminates normally.
constexpr int BLD = NB + 1;    // LDS row stride (floats)

// value of lane LANE of the same row of 16 lanes (DPP row broadcast, folds into the consumer)
template <int LANE>
__device__ inline float row_bcast(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x150 + LANE,
                                                                0xf, 0xf, true));
}

// acc += bcast * y, where bcast is x of lane LANE of the same row of 16 lanes: one VOP2 DPP
// instruction.  The caller separates the write of x from the first such read by two wait
// states (dpp_wait), which the compiler does not do for inline assembly.
template <int LANE>
__device__ inline void fmac_row_bcast(float& acc, float x, float y) {
  asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
               : "+v"(acc) : "v"(x), "v"(y), "n"(LANE));
}
// two wait states between the (earlier) write of v and its (later) DPP reads
__device__ inline void dpp_wait(float& v) { asm volatile("s_nop 1" : "+v"(v)); }

template <int K, int C>
struct LeafCols {
  static __device__ inline void update(float (&a)[16], float lk, float nlk) {
    fmac_row_bcast<C>(a[C], lk, nlk);               // a[C] -= L[C][K] * L[r][K]
    LeafCols<K, C + 1>::update(a, lk, nlk);
  }
};
template <int K>
struct LeafCols<K, 16> {
  static __device__ inline void update(float (&)[16], float, float) {}
};

template <int K>
struct LeafSteps {
  // branch-free: a bad pivot (not positive, or not finite) is replaced by 1 and the first
  // such column of the leaf is remembered in badk
  static __device__ inline void run(float (&a)[16], float (&rsv)[16], int r, int& badk, float thr) {
    dpp_wait(a[K]);                                   // written by the previous step's DPP FMA
    float piv = row_bcast<K>(a[K]);
    const bool bad = !(piv > row_bcast<K>(thr)) || !(piv < 3.0e38f);
    badk = (bad && badk == 16) ? K : badk;
    piv = bad ? 1.f : piv;
    const float rs = __builtin_amdgcn_rsqf(piv);      // 1 ulp
    rsv[K] = rs;
    const float akk = (bad && r == K) ? 1.f : a[K];
    float lk = (r >= K) ? akk * rs : 0.f;             // L[r][K]; row K gets piv * rs = sqrt(piv)
    a[K] = lk;
    const float nlk = -lk;
    dpp_wait(lk);
    LeafCols<K, K + 1>::update(a, lk, nlk);
    LeafSteps<K + 1>::run(a, rsv, r, badk, thr);
  }
};
template <>
struct LeafSteps<16> {
  static __device__ inline void run(float (&)[16], float (&)[16], int, int&, float) {}
};

// Forward substitution L x = e_j with one column j per lane: once x[K] is known every later
// row's running sum takes its term, s[RR] -= L[RR][K] x[K] (independent instructions).
template <int K, int RR>
struct LeafInvRows {
  static __device__ inline void update(const float (&a)[16], float (&sv)[16], float nx) {
    fmac_row_bcast<RR>(sv[RR], a[K], nx);            // a[K] of lane RR is L[RR][K]
    LeafInvRows<K, RR + 1>::update(a, sv, nx);
  }
};
template <int K>
struct LeafInvRows<K, 16> {
  static __device__ inline void update(const float (&)[16], float (&)[16], float) {}
};
template <int K>
struct LeafInv {
  static __device__ inline void run(const float (&a)[16], const float (&rsv)[16], float (&sv)[16]) {
    sv[K] *= rsv[K];                                 // x[K]
    const float nx = -sv[K];
    LeafInvRows<K, K + 1>::update(a, sv, nx);
    LeafInv<K + 1>::run(a, rsv, sv);
  }
};
template <>
struct LeafInv<16> {
  static __device__ inline void run(const float (&)[16], const float (&)[16], float (&)[16]) {}
};

// rows o .. o+15 of M, wavefront 0 only: every row of 16 lanes works on the same leaf (lane
// l holds matrix row l % 16, its 16 columns in registers); lanes 0..15 store the result.
// Pivots and multipliers travel between lanes by DPP row broadcasts.
__device__ inline void factor_leaf(float (*M)[BLD], float (*Inv)[BLD], int o, int nb, int64_t k0,
                                   int* __restrict__ info, const float* __restrict__ thr) {
  const int lane = threadIdx.x & 63, r = lane & 15;
  float a[16], rsv[16], x[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) a[c] = M[o + r][o + c];
  // lane r holds the threshold of the leaf's column r (0 for the identity padding beyond nb)
  float th = (o + r < nb) ? thr[k0 + o + r] : 0.f;
  dpp_wait(th);
  int badk = 16;
  LeafSteps<0>::run(a, rsv, r, badk, th);
  if (badk < 16 && lane == 0 && o + badk < nb) atomicCAS(info, 0, (int)(k0 + o + badk + 1));
  // inverse of the leaf factor: lane j solves L x = e_j
#pragma unroll
  for (int c = 0; c < 16; ++c) x[c] = (c == r) ? 1.f : 0.f;
  LeafInv<0>::run(a, rsv, x);
  if (lane < 16) {
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      M[o + r][o + c] = a[c];
      Inv[o + c][o + r] = x[c];
    }
  }
}

// M: the block (lower triangle meaningful on entry, identity beyond nb); on exit its lower
// triangle is the factor (strict upper part of the leaves zero) and Inv its inverse (lower).
// Tmp is scratch.  256 threads; ends with a barrier.  The 16 x 16 leaf products run on the
// matrix cores (v_mfma_f32_16x16x4_f32: lane l supplies A[l % 16][l / 16] and
// B[l / 16][l % 16] and receives D[4 (l / 16) + r][l % 16], r = 0..3).
__device__ inline void factor_block(float (*M)[BLD], float (*Inv)[BLD], float (*Tmp)[BLD], int nb,
                                    int64_t k0, int* __restrict__ info, const float* __restrict__ thr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lm = lane & 15, lk = lane >> 4;
  for (int e = tid; e < NB * NB; e += 256) Inv[e >> 6][e & 63] = 0.f;
  __syncthreads();
  for (int kb = 0; kb < 4; ++kb) {
    const int o = 16 * kb;
    if (wave == 0) factor_leaf(M, Inv, o, nb, k0, info, thr);
    __syncthreads();
    const int tiles = 3 - kb;             // 16-row tiles under the leaf
    // (b) P = A21 * inv(L11)^T, one row tile per wavefront, in place (a wavefront reads only
    // its own rows of M before it writes them)
    if (wave < tiles) {
      const int r0 = o + 16 + 16 * wave;
      floatx4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 16; kk += 4)
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(M[r0 + lm][o + kk + lk], Inv[o + lm][o + kk + lk], d, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) M[r0 + 4 * lk + r][o + lm] = d[r];
    }
    __syncthreads();
    // (c) A22 -= P P^T on the leaf tiles (ti, tj), tj <= ti
    for (int t = wave; t < tiles * (tiles + 1) / 2; t += 4) {
      int ti = 0;
      while ((ti + 1) * (ti + 2) / 2 <= t) ++ti;
      const int tj = t - ti * (ti + 1) / 2;
      const int r0 = o + 16 + 16 * ti, c0 = o + 16 + 16 * tj;
      floatx4 d;
#pragma unroll
      for (int r = 0; r < 4; ++r) d[r] = M[r0 + 4 * lk + r][c0 + lm];
#pragma unroll
      for (int kk = 0; kk < 16; kk += 4)
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(-M[r0 + lm][o + kk + lk], M[c0 + lm][o + kk + lk], d, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) M[r0 + 4 * lk + r][c0 + lm] = d[r];
    }
    __syncthreads();
  }
  // inverse of the 64 x 64 factor: Inv_ij = -Inv_ii * sum_{k=j}^{i-1} L_ik Inv_kj for i - j = d,
  // one leaf (i, j) per wavefront and level
  for (int d = 1; d < 4; ++d) {
    const int j = wave, i = wave + d;
    if (i < 4) {
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      for (int q = 16 * j; q < 16 * i; q += 4)
        t = __builtin_amdgcn_mfma_f32_16x16x4f32(M[16 * i + lm][q + lk], Inv[q + lk][16 * j + lm], t, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) Tmp[16 * i + 4 * lk + r][16 * j + lm] = t[r];
      // same wavefront reads it back as the right operand (LDS operations of a wavefront are in order)
      floatx4 x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 16; kk += 4)
        x = __builtin_amdgcn_mfma_f32_16x16x4f32(-Inv[16 * i + lm][16 * i + kk + lk], Tmp[16 * i + kk + lk][16 * j + lm], x, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) Inv[16 * i + 4 * lk + r][16 * j + lm] = x[r];
    }
    __syncthreads();
  }
}

// acc (a 16 x 64 strip: rows 16 wave .., tile t = columns 16 t ..) += sign * A B^T over K
// columns, A and B row-major in LDS with odd strides (conflict-free operand reads).
__device__ inline void strip_mma(floatx4 (&acc)[4], const float* __restrict__ A, int lda,
                                 const float* __restrict__ B, int ldb, int K, int wave, int lm, int lk,
                                 float sign) {
  for (int k4 = 0; k4 < K; k4 += 4) {
    const float av = sign * A[(16 * wave + lm) * lda + k4 + lk];
#pragma unroll
    for (int t = 0; t < 4; ++t)
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, B[(16 * t + lm) * ldb + k4 + lk], acc[t], 0, 0, 0);
  }
}

constexpr int PLD = 3 * NB + 1;   // LDS stride of the diagonal rows' earlier columns

// Inner block at columns c0 .. c0 + nb of the outer panel that starts at column J.
// Workgroup w owns rows c0 + 64 + 64 w .. (if any); workgroup 0 also stores the diagonal block.
__global__ __launch_bounds__(256) void chol_panel_kernel(const float* __restrict__ W, float* __restrict__ L,
                                                         int64_t ldl, int64_t n, int64_t J, int64_t c0,
                                                         int nb, int* __restrict__ info,
                                                         const float* __restrict__ thr) {
  extern __shared__ __attribute__((aligned(16))) float psm[];
  float (*M)[BLD] = reinterpret_cast<float (*)[BLD]>(psm);
  float (*Inv)[BLD] = reinterpret_cast<float (*)[BLD]>(psm + NB * BLD);
  float (*Tmp)[BLD] = reinterpret_cast<float (*)[BLD]>(psm + 2 * NB * BLD);
  float (*Po)[BLD] = reinterpret_cast<float (*)[BLD]>(psm + 3 * NB * BLD);
  float (*Pd)[PLD] = reinterpret_cast<float (*)[PLD]>(psm + 4 * NB * BLD);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lm = lane & 15, lk = lane >> 4;
  const int Kp = (int)(c0 - J);               // columns of this panel already factored: 0, 64, 128, 192

  // raw diagonal block (identity beyond nb, strict upper part zero) and the diagonal rows'
  // earlier columns of L; all loads are issued before the first use
  {
    float ld[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u, rr = e >> 6, cc = e & 63;
      const bool in = rr < nb && cc <= rr;
      const float v = W[(c0 + (in ? rr : 0)) * n + c0 + (in ? cc : 0)];
      ld[u] = in ? v : ((rr == cc) ? 1.f : 0.f);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u;
      M[e >> 6][e & 63] = ld[u];
    }
  }
  for (int kc = 0; kc < Kp; kc += NB) {
    float ld[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u, rr = e >> 6, cc = e & 63;
      const float v = L[(c0 + (rr < nb ? rr : 0)) * ldl + J + kc + cc];
      ld[u] = rr < nb ? v : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u;
      Pd[e >> 6][kc + (e & 63)] = ld[u];
    }
  }
  __syncthreads();
  // diagonal block -= (earlier columns) (earlier columns)^T; a wavefront touches its 16 rows only
  if (Kp > 0) {
    floatx4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[t][r] = M[16 * wave + 4 * lk + r][16 * t + lm];
    strip_mma(acc, &Pd[0][0], PLD, &Pd[0][0], PLD, Kp, wave, lm, lk, -1.f);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) M[16 * wave + 4 * lk + r][16 * t + lm] = acc[t][r];
  }
  __syncthreads();
  factor_block(M, Inv, Tmp, nb, c0, info, thr);
  if (blockIdx.x == 0) {
    for (int e = tid; e < NB * NB; e += 256) {
      const int rr = e >> 6, cc = e & 63;
      if (rr < nb && cc <= rr) L[(c0 + rr) * ldl + c0 + cc] = M[rr][cc];
    }
  }
  const int64_t r0 = c0 + NB + (int64_t)blockIdx.x * NB;
  if (r0 >= n) return;
  // own rows: X = W[rows, block] - L[rows, earlier columns] (diagonal rows' earlier columns)^T
  floatx4 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = r0 + 16 * wave + 4 * lk + r;
      const int col = 16 * t + lm;
      acc[t][r] = (row < n && col < nb) ? W[row * n + c0 + col] : 0.f;
    }
  for (int kc = 0; kc < Kp; kc += NB) {
    float ld[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u, rr = e >> 6, cc = e & 63;
      const bool in = r0 + rr < n;
      const float v = L[(r0 + (in ? rr : 0)) * ldl + J + kc + cc];
      ld[u] = in ? v : 0.f;
    }
    __syncthreads();                    // the previous chunk has been consumed
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = tid + 256 * u;
      Po[e >> 6][e & 63] = ld[u];
    }
    __syncthreads();
    strip_mma(acc, &Po[0][0], BLD, &Pd[0][kc], PLD, NB, wave, lm, lk, -1.f);
  }
  // rows = X inv(factor)^T; X goes through LDS to become the left operand (each wavefront
  // reads back only the 16 rows it wrote)
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) Tmp[16 * wave + 4 * lk + r][16 * t + lm] = acc[t][r];
  floatx4 out[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) out[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  strip_mma(out, &Tmp[0][0], BLD, &Inv[0][0], BLD, NB, wave, lm, lk, 1.f);
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = r0 + 16 * wave + 4 * lk + r;
      const int col = 16 * t + lm;
      if (row < n && col < nb) L[row * ldl + c0 + col] = out[t][r];
    }
}

}  // namespace

constexpr int kOuter = 4 * NB;
constexpr int kPanelLds = (4 * NB * BLD + NB * PLD) * (int)sizeof(float);

size_t cholesky_scratch_bytes(int64_t n) {
  return kAlign + 2 * align_up((size_t)n * sizeof(float)) + align_up((size_t)n * n * sizeof(float));
}

hipError_t launch_cholesky(hipStream_t s, const float* H, int64_t n, int64_t ldh, int precond,
                           float lambda, float* L, int64_t ldl, int* info_dev) {
  // info_dev points at scratch: [int info][pad to 256][float delta[n]][float thr[n]][float W[n x n]]
  float* delta = reinterpret_cast<float*>(reinterpret_cast<char*>(info_dev) + kAlign);
  float* thr = reinterpret_cast<float*>(reinterpret_cast<char*>(delta) + align_up((size_t)n * sizeof(float)));
  float* W = reinterpret_cast<float*>(reinterpret_cast<char*>(thr) + align_up((size_t)n * sizeof(float)));
  // A pivot at or below tau times its column's diagonal entry is rounding noise of the fp32
  // Schur complement (about sqrt(n) 2^-24 of that entry), not information: the matrix is then
  // numerically singular and the factor would be useless to the S-update.
  const float tau = 8.f * sqrtf((float)n) * 5.9604645e-8f;
  hipError_t e;
  static std::atomic<uint64_t> lds_set{0};
  if ((e = ensure_dynamic_lds((const void*)chol_panel_kernel, kPanelLds, lds_set)) != hipSuccess) return e;
  hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(1), 0, s, info_dev, 0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (precond == GANQ_PRECOND_DIAGDOM) {
    hipLaunchKernelGGL(diagdom_delta_kernel, dim3((unsigned)n), dim3(256), 0, s, H, n, ldh, delta);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const bool vec = (n % 4) == 0 && (ldh % 4) == 0 && (ldl % 4) == 0 && (((uintptr_t)H | (uintptr_t)L) & 15) == 0;
  const dim3 cgrid((unsigned)ceil_div(n, 1024), (unsigned)n);
  if (vec)
    hipLaunchKernelGGL(copy_lower_kernel<true>, cgrid, dim3(256), 0, s, H, n, ldh, W, L, ldl, precond, lambda,
                       delta, tau, thr);
  else
    hipLaunchKernelGGL(copy_lower_kernel<false>, cgrid, dim3(256), 0, s, H, n, ldh, W, L, ldl, precond, lambda,
                       delta, tau, thr);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  for (int64_t J = 0; J < n; J += kOuter) {
    for (int64_t c0 = J; c0 < n && c0 < J + kOuter; c0 += NB) {
      const int nb = (int)((n - c0 < NB) ? n - c0 : NB);
      const int64_t rem = n - c0 - NB;
      const unsigned wgs = rem > 0 ? (unsigned)ceil_div(rem, NB) : 1u;
      hipLaunchKernelGGL(chol_panel_kernel, dim3(wgs), dim3(256), kPanelLds, s, W, L, ldl, n, J, c0, nb,
                         info_dev, thr);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const int64_t rem = n - J - kOuter;
    if (rem <= 0) break;
    // W22 -= L21 L21^T, lower tiles only
    const float* L21 = L + (J + kOuter) * ldl + J;
    float* W22 = W + (J + kOuter) * n + (J + kOuter);
    if ((ldl % 4) == 0 && (((uintptr_t)L21) % 16) == 0 && 128 * ldl * 4 < ((int64_t)1 << 31))
      e = launch_syrk256_f32(s, rem, L21, ldl, W22, n);
    else
      e = launch_gemm_f32(s, /*transb=*/1, /*lower_only=*/1, rem, rem, kOuter, -1.f, L21, ldl, L21, ldl, 1.f, W22, n);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ganq
