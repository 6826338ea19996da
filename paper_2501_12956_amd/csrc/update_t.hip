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
// LDS (dynamic): two stages of { A hi tile, A lo tile, one-hot B tile } and the per-wavefront
// fold accumulators.  The one-hot tile is never rebuilt: it starts as zeros and each thread
// owns a fixed set of (row i, k) positions whose single 1 it moves - it clears the 1 it
// wrote when the stage was last used and sets the new one (in-order LDS writes of one
// thread), so staging B costs a few 16-bit LDS writes instead of a compare per element.
constexpr int T_STAGE_BYTES = 2 * TM * TLD * 2 + TN * TLD * 2;
constexpr int T_NSTAGE = 1;   // one LDS stage: two barriers per k-step, two workgroups per CU

template <int NBITS>
__global__ __launch_bounds__(256) void t_accum_kernel(const _Float16* __restrict__ Hhi,
                                                      const _Float16* __restrict__ Hlo,
                                                      int64_t npad, const uint8_t* __restrict__ Qp,
                                                      int64_t mpad, int mtiles,
                                                      float* __restrict__ Apart) {
  constexpr int C = 1 << NBITS;
  constexpr int RW = TN >> NBITS;             // rows i per workgroup
  constexpr int EPT = (RW * TK) / 256;        // (i, k) positions per thread and stage: 32 >> NBITS
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto As_hi = [&](int st) { return reinterpret_cast<_Float16 (*)[TLD]>(smem + st * T_STAGE_BYTES); };
  auto As_lo = [&](int st) { return reinterpret_cast<_Float16 (*)[TLD]>(smem + st * T_STAGE_BYTES + TM * TLD * 2); };
  auto Bs_of = [&](int st) { return reinterpret_cast<_Float16 (*)[TLD]>(smem + st * T_STAGE_BYTES + 2 * TM * TLD * 2); };
  float* Aw = reinterpret_cast<float*>(smem + T_NSTAGE * T_STAGE_BYTES);        // [4][128*C]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int kh = lane >> 5, l32 = lane & 31;
  const int64_t i0 = (int64_t)blockIdx.x * RW;
  const int group = blockIdx.y;

  for (int e = tid; e < 4 * 128 * C; e += 256) Aw[e] = 0.f;
  for (int st = 0; st < T_NSTAGE; ++st) {
    _Float16* bz = &Bs_of(st)[0][0];
    for (int e = tid; e < TN * TLD / 8; e += 256) reinterpret_cast<uint4*>(bz)[e] = uint4{0u, 0u, 0u, 0u};
  }

  // one-hot staging: this thread owns row il and the EPT consecutive k from kk0 of every stage
  const int ex_il = (tid * EPT) / TK, ex_kk0 = (tid * EPT) % TK;
  const uint8_t* __restrict__ qrow = Qp + (i0 + ex_il) * npad + ex_kk0;
  int old_code[1][EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) old_code[0][e] = -1;
  const int lrow = tid >> 2, lk = (tid & 3) * 8;
  __syncthreads();

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

    // Global operands are fetched two k-steps ahead into two alternating register sets: a
    // set is written to LDS at the top of its k-step and refilled right away for the k-step
    // after next, so a load has two MFMA sections to complete.
    struct Regs {
      half8 hi[2], lo[2];
      uint8_t q[EPT];
    };
    auto fetch = [&](Regs& r, int64_t k0) {
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        const int64_t off = (jt0 + lrow + 64 * ps) * npad + k0 + lk;
        r.hi[ps] = *reinterpret_cast<const half8*>(Hhi + off);
        r.lo[ps] = *reinterpret_cast<const half8*>(Hlo + off);
      }
      if constexpr (EPT == 2) {
        const uint16_t w = *reinterpret_cast<const uint16_t*>(qrow + k0);
        r.q[0] = (uint8_t)(w & 0xff); r.q[1] = (uint8_t)(w >> 8);
      } else if constexpr (EPT == 4) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(qrow + k0);
#pragma unroll
        for (int e = 0; e < 4; ++e) r.q[e] = (uint8_t)((w >> (8 * e)) & 0xff);
      } else {
#pragma unroll
        for (int e = 0; e < EPT; ++e) r.q[e] = qrow[k0 + e];
      }
    };
    _Float16 (*AsHi)[TLD] = As_hi(0);
    _Float16 (*AsLo)[TLD] = As_lo(0);
    _Float16 (*Bs)[TLD] = Bs_of(0);
    auto kstep = [&](Regs& r, int64_t k0) {
      __syncthreads();                      // every wavefront is done reading the previous stage
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        *reinterpret_cast<half8*>(&AsHi[lrow + 64 * ps][lk]) = r.hi[ps];
        *reinterpret_cast<half8*>(&AsLo[lrow + 64 * ps][lk]) = r.lo[ps];
      }
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int code = r.q[e] & (C - 1);
        if (old_code[0][e] >= 0) Bs[ex_il * C + old_code[0][e]][ex_kk0 + e] = (_Float16)0;
        Bs[ex_il * C + code][ex_kk0 + e] = (_Float16)1;
        old_code[0][e] = code;
      }
      __syncthreads();
      if (k0 + 2 * TK < kend) fetch(r, k0 + 2 * TK);
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
    };
    Regs r0, r1;
    fetch(r0, 0);
    if (TK < kend) fetch(r1, TK);
    for (int64_t k0 = 0; k0 < kend; k0 += 2 * TK) {     // kend is a multiple of 2 TK (TM = 4 TK)
      kstep(r0, k0);
      kstep(r1, k0 + TK);
    }

    // fold: Z[j, (il, b)] -> Aw[wave][il_w][Q[i][j]][b].  The codes of this lane's 32 rows j
    // are fetched first (8 dwords per row i), so that the loads overlap instead of each
    // waiting behind an LDS add.
    float* __restrict__ myA = Aw + wave * 128 * C;
    uint32_t qd[4][2][4];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int ilw = (ni * 32 + l32) >> NBITS;
      const uint8_t* __restrict__ qr = Qp + (i0 + wc * (RW >> 1) + ilw) * npad + jt0 + wr * 64;
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
          qd[ni][mi][vq] = *reinterpret_cast<const uint32_t*>(qr + mi * 32 + vq * 8 + kh * 4);
    }
    // LDS float atomics are serialised lane by lane on this chip, so the adds are plain
    // read-modify-writes instead: in each of two passes only the lanes of one half (kh) are
    // active, which makes every active lane's bin (its own column (il, b), any code a) private
    // to it; LDS operations of one wavefront execute in program order, so a later step sees
    // the earlier one's write.  The four column tiles (ni) form independent streams.
    int base[4];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int colw = ni * 32 + l32;                 // pair index within this wave's 128
      base[ni] = (colw >> NBITS) * C * C + (colw & (C - 1));
    }
    for (int pass = 0; pass < 2; ++pass) {
      if (kh == pass) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            // register v of the tile is row mi*32 + (v>>2)*8 + kh*4 + (v&3) of this wave's 64
            float x[4];
            int ad[4];
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
              const int a = (qd[ni][mi][v >> 2] >> (8 * (v & 3))) & (C - 1);
              ad[ni] = base[ni] + a * C;
              x[ni] = myA[ad[ni]];
            }
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) myA[ad[ni]] = x[ni] + acc[mi][ni][v];
          }
      }
    }
    // the stage that the next row tile writes first may still be read by slower wavefronts
    __syncthreads();
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

  // per-code sums over the row: lane l takes columns l, l + 64, ... (coalesced) and adds into
  // its own column of LDS bins; the 64 partial sums per code are then added in a fixed order
  __shared__ float binD[16][64], binB[16][64];
  __shared__ int binC[16][64];
  for (int a = 0; a < C; ++a) {
    binD[a][tid] = 0.f;
    binB[a][tid] = 0.f;
    binC[a][tid] = 0;
  }
  for (int64_t j = tid; j < n; j += 64) {
    const int a = Q[i * ldq + j] & (C - 1);
    binD[a][tid] += Hdiag[j];      // lane-private bins: plain read-modify-write
    binB[a][tid] += G[i * ldg + j];
    binC[a][tid] += 1;
  }
  __syncthreads();
  if (tid < C) {
    double sd = 0.0, sb = 0.0;
    int c0 = 0;
    for (int l = 0; l < 64; ++l) {
      sd += (double)binD[tid][l];
      sb += (double)binB[tid][l];
      c0 += binC[tid][l];
    }
    Dg[tid] = sd;
    rhs[tid] = sb;
    cnt[tid] = c0;
    dead[tid] = (c0 == 0);
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
template <int NBITS>
static hipError_t launch_t_accum_n(hipStream_t s, int64_t m, int64_t n, void* scratch) {
  TScratch sc;
  t_layout(m, n, NBITS, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, NBITS);
  const int C = 1 << NBITS;
  const int mtiles = (int)(npad / TM);
  const int groups = t_groups(n);
  const size_t shmem = T_NSTAGE * T_STAGE_BYTES + 4 * 128 * C * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)t_accum_kernel<NBITS>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(t_accum_kernel<NBITS>, dim3((unsigned)(mpad / (TN >> NBITS)), (unsigned)groups),
                     dim3(256), shmem, s, sc.Hhi, sc.Hlo, npad, sc.Qp, mpad, mtiles, sc.Apart);
  return hipGetLastError();
}

hipError_t launch_t_accum(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch) {
  switch (nbits) {
    case 1: return launch_t_accum_n<1>(s, m, n, scratch);
    case 2: return launch_t_accum_n<2>(s, m, n, scratch);
    case 3: return launch_t_accum_n<3>(s, m, n, scratch);
    default: return launch_t_accum_n<4>(s, m, n, scratch);
  }
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
