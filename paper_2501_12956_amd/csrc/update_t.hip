// T-update of GANQ: T_i = W_i H S_i^T (S_i H S_i^T)^dagger per row, Eq. (4)-(7).
//
// A_i = S_i H S_i^T is a C x C matrix whose entry (a, b) is the sum of H_jk over
// the columns j with code a and k with code b; b_i = S_i (W H)_i^T sums the
// entries of G = W H by code.  Forming A_i costs n^2 additions per row however
// it is arranged.  Here the additions run on the matrix cores:
//
//   Z[j, (i,b)] = sum_{k<j} H_jk [Q_ik == b]
//
// is a GEMM whose left operand is the strictly lower triangle of H and whose
// right operand is the one-hot expansion of Q, generated on the fly from the
// index bytes.  One-hot entries are exact in fp16; H is split into two fp16
// pieces (hi + lo, 22 significant bits, pre-scaled by a power of two so that the
// largest entry sits near 2^15), both accumulated in fp32 by
// v_mfma_f32_32x32x16_f16.  Only k < j is visited (H is symmetric):
//   M_i[a, b] = sum_j [Q_ij == a] Z[j, (i,b)],   A_i = M_i + M_i^T + Diag(D_i),
//   D_i[a] = sum_{j: Q_ij == a} H_jj.
// The fold over j is done in the GEMM epilogue with LDS adds into per-wavefront
// copies (fixed order, no global float atomics); partial M_i per group of row
// tiles of H go to scratch and are summed in float64 by the solve kernel, which
// also forms D_i and b_i, drops unused codes (pseudo-inverse reading: their
// entry is 0, or kept) and solves the reduced system by Cholesky in float64.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int TM = 128;    // rows j of H per tile
constexpr int TN = 256;    // (row i, code b) pairs per workgroup
constexpr int TK = 32;     // k per stage
constexpr int TPAD = 8;    // halfs of LDS row padding
constexpr int TLD = TK + TPAD;

// ---- per-layer preparation: fp16 hi/lo split of the strictly lower triangle of H ----
__global__ __launch_bounds__(256) void maxdiag_kernel(const float* __restrict__ H, int64_t n,
                                                      int64_t ldh, float* __restrict__ scale,
                                                      float* __restrict__ Hdiag) {
  __shared__ float red[256];
  float mx = 0.f;
  for (int64_t j = threadIdx.x; j < n; j += 256) {
    const float d = H[j * ldh + j];
    Hdiag[j] = d;
    const float ad = fabsf(d);
    if (ad < __builtin_huge_valf() && ad > mx) mx = ad;
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float s = 1.f;
    if (red[0] > 0.f) s = ldexpf(1.f, 14 - ilogbf(red[0]));   // max * s in [2^14, 2^15)
    scale[0] = s;
    scale[1] = 1.f / s;
  }
}

__global__ __launch_bounds__(256) void split_lower_kernel(const float* __restrict__ H, int64_t n,
                                                          int64_t ldh, int64_t npad,
                                                          const float* __restrict__ scale,
                                                          _Float16* __restrict__ Hhi,
                                                          _Float16* __restrict__ Hlo) {
  const int64_t j = blockIdx.y;                                   // row of H
  const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;      // column
  if (k >= npad) return;
  // only tiles that the GEMM reads: k-tile <= j-tile (tiles of TM)
  if (k / TM > j / TM) return;
  _Float16 hi = (_Float16)0, lo = (_Float16)0;
  if (j < n && k < j) {
    const float v = H[j * ldh + k] * scale[0];
    hi = (_Float16)v;
    lo = (_Float16)(v - (float)hi);
  }
  Hhi[j * npad + k] = hi;
  Hlo[j * npad + k] = lo;
}

// zero-padded, 16-byte aligned copy of Q
__global__ __launch_bounds__(256) void pad_q_kernel(const uint8_t* __restrict__ Q, int64_t m,
                                                    int64_t n, int64_t ldq, int64_t npad,
                                                    uint8_t* __restrict__ Qp) {
  const int64_t i = blockIdx.y;
  const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (k >= npad) return;
  Qp[i * npad + k] = (i < m && k < n) ? Q[i * ldq + k] : (uint8_t)0;
}

// ---- the GEMM with fold epilogue ----
__global__ __launch_bounds__(256) void t_accum_kernel(const _Float16* __restrict__ Hhi,
                                                      const _Float16* __restrict__ Hlo,
                                                      int64_t npad, const uint8_t* __restrict__ Qp,
                                                      int64_t mpad, int nbits, int mtiles,
                                                      float* __restrict__ Apart) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16 (*AsHi)[TLD] = reinterpret_cast<_Float16 (*)[TLD]>(smem);
  _Float16 (*AsLo)[TLD] = reinterpret_cast<_Float16 (*)[TLD]>(smem + TM * TLD * 2);
  _Float16 (*Bs)[TLD] = reinterpret_cast<_Float16 (*)[TLD]>(smem + 2 * TM * TLD * 2);
  float* Aw = reinterpret_cast<float*>(smem + 2 * TM * TLD * 2 + TN * TLD * 2);  // [4][128*C]

  const int C = 1 << nbits;
  const int RW = TN >> nbits;                 // rows i per workgroup
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int kh = lane >> 5, l32 = lane & 31;
  const int64_t i0 = (int64_t)blockIdx.x * RW;
  const int group = blockIdx.y;

  for (int e = tid; e < 4 * 128 * C; e += 256) Aw[e] = 0.f;

  // one-hot expansion: this thread owns pair (il, b) and all TK k of a stage
  const int ex_il = tid >> nbits, ex_b = tid & (C - 1);
  const uint8_t* __restrict__ qrow = Qp + (i0 + ex_il) * npad;
  const int lrow = tid >> 2, lk = (tid & 3) * 8;

  for (int half = 0; half < 2; ++half) {
    const int mt = (half == 0) ? group : mtiles - 1 - group;
    if (half == 1 && mt == group) break;
    const int64_t jt0 = (int64_t)mt * TM;
    const int64_t kend = jt0 + TM;            // tiles right of the diagonal are never needed

    floatx16 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    half8 rhi[2], rlo[2];
    uint4 rq[2];
    auto fetch = [&](int64_t k0) {
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        const int64_t off = (jt0 + lrow + 64 * ps) * npad + k0 + lk;
        rhi[ps] = *reinterpret_cast<const half8*>(Hhi + off);
        rlo[ps] = *reinterpret_cast<const half8*>(Hlo + off);
      }
      rq[0] = *reinterpret_cast<const uint4*>(qrow + k0);
      rq[1] = *reinterpret_cast<const uint4*>(qrow + k0 + 16);
    };

    fetch(0);
    for (int64_t k0 = 0; k0 < kend; k0 += TK) {
      __syncthreads();
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        *reinterpret_cast<half8*>(&AsHi[lrow + 64 * ps][lk]) = rhi[ps];
        *reinterpret_cast<half8*>(&AsLo[lrow + 64 * ps][lk]) = rlo[ps];
      }
#pragma unroll
      for (int w4 = 0; w4 < 2; ++w4) {
        const uint32_t words[4] = {rq[w4].x, rq[w4].y, rq[w4].z, rq[w4].w};
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          half8 oh;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t wd = words[hh * 2 + (e >> 2)];
            const int code = (wd >> (8 * (e & 3))) & 0xff;
            oh[e] = (code == ex_b) ? (_Float16)1 : (_Float16)0;
          }
          *reinterpret_cast<half8*>(&Bs[tid][w4 * 16 + hh * 8]) = oh;
        }
      }
      __syncthreads();
      if (k0 + TK < kend) fetch(k0 + TK);
#pragma unroll
      for (int ks = 0; ks < TK; ks += 16) {
        half8 ahi[2], alo[2], bf[4];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
          ahi[mi] = *reinterpret_cast<const half8*>(&AsHi[wr * 64 + mi * 32 + l32][ks + 8 * kh]);
          alo[mi] = *reinterpret_cast<const half8*>(&AsLo[wr * 64 + mi * 32 + l32][ks + 8 * kh]);
        }
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
          bf[ni] = *reinterpret_cast<const half8*>(&Bs[wc * 128 + ni * 32 + l32][ks + 8 * kh]);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int ni = 0; ni < 4; ++ni) {
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi[mi], bf[ni], acc[mi][ni], 0, 0, 0);
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo[mi], bf[ni], acc[mi][ni], 0, 0, 0);
          }
      }
    }

    // fold: Z[j, (il, b)] -> Aw[wave][il_w][Q[i][j]][b]
    float* __restrict__ myA = Aw + wave * 128 * C;
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int colw = ni * 32 + l32;                 // pair index within this wave's 128
      const int ilw = colw >> nbits, b = colw & (C - 1);
      const uint8_t* __restrict__ qr = Qp + (i0 + wc * (RW >> 1) + ilw) * npad + jt0 + wr * 64;
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int jl = mi * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
          const int a = qr[jl] & (C - 1);
          atomicAdd(&myA[(ilw * C + a) * C + b], acc[mi][ni][v]);
        }
    }
  }
  __syncthreads();
  // Apart[group][i][a*C + b] = copy(wr = 0) + copy(wr = 1)
  const int per_half = (RW >> 1) * C * C;    // = 128 * C
  for (int e = tid; e < RW * C * C; e += 256) {
    const int wcx = e / per_half, rem = e % per_half;
    const float v = Aw[(0 * 2 + wcx) * 128 * C + rem] + Aw[(1 * 2 + wcx) * 128 * C + rem];
    Apart[((int64_t)group * mpad + i0) * C * C + e] = v;
  }
}

// ---- per-row assembly and solve (one wavefront per row, float64) ----
__global__ __launch_bounds__(64) void t_solve_kernel(const float* __restrict__ Apart, int ngroups,
                                                     int64_t mpad, const float* __restrict__ scale,
                                                     const float* __restrict__ Hdiag,
                                                     const float* __restrict__ G, int64_t ldg,
                                                     const uint8_t* __restrict__ Q, int64_t ldq,
                                                     int64_t n, int nbits, int empty_mode,
                                                     float* __restrict__ T,
                                                     int32_t* __restrict__ empty_count) {
  __shared__ double A[16][17];
  __shared__ double rhs[16], Dg[16], diag0[16];
  __shared__ int cnt[16], dead[16];
  const int C = 1 << nbits;
  const int64_t i = blockIdx.x;
  const int tid = threadIdx.x;

  // per-code sums over the row: lane = 4 * code + part, each part strides over j
  {
    const int a = tid >> 2, part = tid & 3;
    double sd = 0.0, sb = 0.0;
    int c0 = 0;
    if (a < C) {
      for (int64_t j = part; j < n; j += 4) {
        if ((Q[i * ldq + j] & (C - 1)) == a) {
          sd += (double)Hdiag[j];
          sb += (double)G[i * ldg + j];
          ++c0;
        }
      }
    }
    // combine the 4 parts in a fixed order
    sd += __shfl_xor(sd, 1, 64); sb += __shfl_xor(sb, 1, 64); c0 += __shfl_xor(c0, 1, 64);
    sd += __shfl_xor(sd, 2, 64); sb += __shfl_xor(sb, 2, 64); c0 += __shfl_xor(c0, 2, 64);
    if (part == 0 && a < C) { Dg[a] = sd; rhs[a] = sb; cnt[a] = c0; dead[a] = (c0 == 0); }
  }
  __syncthreads();
  const double inv_s = (double)scale[1];
  for (int e = tid; e < C * C; e += 64) {
    const int a = e / C, b = e % C;
    double lo = 0.0, up = 0.0;
    for (int g = 0; g < ngroups; ++g) {
      const float* __restrict__ P = Apart + ((int64_t)g * mpad + i) * C * C;
      lo += (double)P[a * C + b];
      up += (double)P[b * C + a];
    }
    double v = (lo + up) * inv_s;
    if (a == b) { v += Dg[a]; diag0[a] = v; }
    A[a][b] = v;
  }
  __syncthreads();
  // in-place Cholesky of the non-empty principal submatrix (lower), column by column
  for (int k = 0; k < C; ++k) {
    if (tid == 0) {
      double d = A[k][k];
      if (!dead[k]) {
        // relative pivot tolerance: a code whose column is numerically dependent is dropped
        if (!(d > 1e-10 * diag0[k]) || !(d < 1.79e308)) dead[k] = 2;
      }
      A[k][k] = dead[k] ? 1.0 : sqrt(d);
    }
    __syncthreads();
    const bool kd = dead[k] != 0;
    const double dk = A[k][k];
    if (tid > k && tid < C) A[tid][k] = (kd || dead[tid]) ? 0.0 : A[tid][k] / dk;
    __syncthreads();
    if (!kd) {
      for (int e = tid; e < C * C; e += 64) {
        const int r = e / C, c = e % C;
        if (c > k && c <= r) A[r][c] -= A[r][k] * A[c][k];
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    double y[16];
    int nempty = 0;
    for (int a = 0; a < C; ++a) {
      double s = dead[a] ? 0.0 : rhs[a];
      for (int q = 0; q < a; ++q) s -= A[a][q] * y[q];
      y[a] = dead[a] ? 0.0 : s / A[a][a];
    }
    for (int a = C - 1; a >= 0; --a) {
      double s = y[a];
      for (int q = a + 1; q < C; ++q) s -= A[q][a] * y[q];
      y[a] = dead[a] ? 0.0 : s / A[a][a];
    }
    for (int a = 0; a < C; ++a) {
      if (dead[a]) {
        ++nempty;
        if (empty_mode == GANQ_EMPTY_ZERO || dead[a] == 2) T[i * C + a] = 0.f;
      } else {
        T[i * C + a] = (float)y[a];
      }
    }
    if (empty_count != nullptr) empty_count[i] = nempty;
  }
}

inline int64_t t_npad(int64_t n) { return ceil_div(n, TM) * TM; }
inline int64_t t_mpad(int64_t m, int nbits) { const int64_t rw = TN >> nbits; return ceil_div(m, rw) * rw; }
inline int t_groups(int64_t n) { return (int)((ceil_div(n, TM) + 1) / 2); }

struct TScratch {
  float* scale;
  float* Hdiag;
  _Float16* Hhi;
  _Float16* Hlo;
  uint8_t* Qp;
  float* Apart;
};

inline size_t t_layout(int64_t m, int64_t n, int nbits, char* base, TScratch* out) {
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  const int C = 1 << nbits;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t o_scale = take(2 * sizeof(float));
  const size_t o_diag = take((size_t)n * sizeof(float));
  const size_t o_hi = take((size_t)npad * npad * sizeof(_Float16));
  const size_t o_lo = take((size_t)npad * npad * sizeof(_Float16));
  const size_t o_q = take((size_t)mpad * npad);
  const size_t o_ap = take((size_t)t_groups(n) * mpad * C * C * sizeof(float));
  if (out != nullptr) {
    out->scale = (float*)(base + o_scale);
    out->Hdiag = (float*)(base + o_diag);
    out->Hhi = (_Float16*)(base + o_hi);
    out->Hlo = (_Float16*)(base + o_lo);
    out->Qp = (uint8_t*)(base + o_q);
    out->Apart = (float*)(base + o_ap);
  }
  return off;
}

}  // namespace

size_t update_t_scratch_bytes(int64_t m, int64_t n, int nbits) {
  return t_layout(m, n, nbits, nullptr, nullptr);
}

// fp16 hi/lo split of the strictly lower triangle of H into scratch (once per layer).
hipError_t launch_t_prepare(hipStream_t s, const float* H, int64_t m, int64_t n, int64_t ldh,
                            int nbits, void* scratch) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n);
  hipLaunchKernelGGL(maxdiag_kernel, dim3(1), dim3(256), 0, s, H, n, ldh, sc.scale, sc.Hdiag);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(split_lower_kernel, dim3((unsigned)ceil_div(npad, 256), (unsigned)npad),
                     dim3(256), 0, s, H, n, ldh, npad, sc.scale, sc.Hhi, sc.Hlo);
  return hipGetLastError();
}

// zero-padded aligned copy of Q into scratch
hipError_t launch_t_pad(hipStream_t s, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                        int nbits, void* scratch) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  hipLaunchKernelGGL(pad_q_kernel, dim3((unsigned)ceil_div(npad, 256), (unsigned)mpad), dim3(256), 0,
                     s, Q, m, n, ldq, npad, sc.Qp);
  return hipGetLastError();
}

// partial M_i = sum_{j>k} [Q_ij = a][Q_ik = b] H_jk per group of row tiles (the one-hot GEMM)
hipError_t launch_t_accum(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  const int C = 1 << nbits;
  const int mtiles = (int)(npad / TM);
  const int groups = t_groups(n);
  const size_t shmem = 2 * TM * TLD * 2 + TN * TLD * 2 + 4 * 128 * C * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)t_accum_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       2 * TM * TLD * 2 + TN * TLD * 2 + 4 * 128 * 16 * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(t_accum_kernel, dim3((unsigned)(mpad / (TN >> nbits)), (unsigned)groups),
                     dim3(256), shmem, s, sc.Hhi, sc.Hlo, npad, sc.Qp, mpad, nbits, mtiles,
                     sc.Apart);
  return hipGetLastError();
}

// assemble A_i, b_i and solve; G = W H
hipError_t launch_t_solve(hipStream_t s, const float* G, int64_t ldg, int64_t m, int64_t n,
                          const uint8_t* Q, int64_t ldq, int nbits, int empty_mode, float* T,
                          int32_t* empty_count, void* scratch) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t mpad = t_mpad(m, nbits);
  hipLaunchKernelGGL(t_solve_kernel, dim3((unsigned)m), dim3(64), 0, s, sc.Apart, t_groups(n), mpad,
                     sc.scale, sc.Hdiag, G, ldg, Q, ldq, n, nbits, empty_mode, T, empty_count);
  return hipGetLastError();
}

}  // namespace ganq
