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
// right operand is the one-hot expansion of Q, kept in LDS and updated in place
// from precomputed positions.  It runs in integer arithmetic on
// v_mfma_i32_32x32x32_i8 (twice the fp16 rate, exact accumulation):
//   H_jk ~ v_jk 2^(e_k - s_j),  v_jk an integer of 16, 24 or 32 bits,
// with a power-of-two column factor 2^e_k (e_k = 0..6, from the diagonal, so that a row's
// entries use the same digits whether their column is large or small; it is the value of
// the one-hot entry, which an int8 operand can hold) and a power-of-two row factor chosen
// so that the row's largest |v| fills the digits.  v is split into balanced base-256 digits,
// one GEMM pass per digit from the top.  Where sum_k |v_jk| 2^e_k < 2^30 for every row of a
// tile of 128 rows (no subset sum can overflow an int32) the digits share the accumulators,
// shifted left by 8 between passes, which end as sum_k v_jk 2^e_k [Q_ik == b] exactly;
// elsewhere each digit is folded on its own.  A tile takes two digits when, for every row,
// 16 times the largest scaled entry stays below sqrt(H_jj) g, g the smallest
// sqrt(H_kk) 2^-e_k over the live columns (about sqrt(max H) / 64 when the columns' scales
// span less than the 2^6 the column factors cover; never taken below 2^-18 sqrt(max H)):
// the absolute error of an entry is then at most 2^-20 sqrt(H_jj H_kk), that of 20-bit
// digits on a fully correlated row.  Otherwise it takes three digits, or four where the same
// bound needs them (feature scales spread over more than 2^10).
// Only k < j is visited (H is symmetric):
//   M_i[a, b] = sum_j [Q_ij == a] Z[j, (i,b)],   A_i = M_i + M_i^T + Diag(D_i),
//   D_i[a] = sum_{j: Q_ij == a} H_jj.
// The fold over j runs on the matrix cores as well, straight from the accumulator
// registers and with the row factor 2^-s_j as the left operand (see t_accum_kernel); partial
// M_i per group of row tiles of H go to scratch and are summed in float64 by the solve
// kernel, which also forms D_i and b_i, drops unused codes (pseudo-inverse reading: their
// entry is 0, or kept) and solves the reduced system by Cholesky in float64.
//
// Later sweeps of Algorithm 1 change few indices (a few per cent from the fifth sweep on the
// synthetic layers), and S_i H0 S_i^T (H0 = H without its diagonal) can then be brought up to
// date instead of being summed again: with D = S_new - S_old (two entries per changed column)
//   A_new - A_old = D (H0 S_new^T) + (D (H0 S_old^T))^T,
// which needs, for each changed column j of row i only, the sums of row j of H0 by the new and by
// the old codes: |changed| n additions per row instead of n^2 / 2.  The rows of H are gathered by
// index, so nothing is shared between the rows of W and the cost is the bytes of H that move: the
// update pays off below about 3.5 % changed indices (t_delta_kernel; the choice is made on the
// device, per sweep, from the counts of the kernel that lists the changes).  The state A_i is kept
// in float64 and every change is an exact integer sum scaled by a power of two.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int TM = 128;    // rows j of H per tile
// Four wavefronts per workgroup, each 128 x 64 of the tile, and two workgroups per compute unit
// (72 KB of LDS each): the two wavefronts that share a SIMD then belong to different workgroups
// and are not held to the same barrier, so one's staging work runs under the other's MFMAs.
constexpr int TNW = 4;
constexpr int TN = 64 * TNW;    // (row i, code b) pairs per workgroup
constexpr int TK = 64;     // k per stage
constexpr int TP = 4;      // most base-256 digits per entry
constexpr int EMAX = 6;    // largest column exponent (the one-hot entry 2^e is an int8)
constexpr float V2MAX = 32512.f;     // largest |v| with two digits:  127 * 256 + 127 - 127
constexpr float V3MAX = 8323072.f;   // with three: 2^23 - 2^16 (four: 256 times that, 2^31 - 2^24)

// ---- per-layer preparation ----
// diagonal of H, column exponents e_k = clamp(EMAX + round(log2 sqrt(H_kk / max H)), 0, EMAX)
// (stored as the one-hot value 2^e_k); the per-tile flags start cleared
__global__ __launch_bounds__(256) void t_diag_kernel(const float* __restrict__ H, int64_t n,
                                                     int64_t ldh, int64_t npad, int mtiles,
                                                     float* __restrict__ scale,
                                                     float* __restrict__ Hdiag,
                                                     uint8_t* __restrict__ Cs, int* __restrict__ Ptile) {
  __shared__ float red[256];
  float mx = 0.f;
  for (int64_t j = threadIdx.x; j < n; j += 256) {
    const float d = H[j * ldh + j];
    Hdiag[j] = d;
    if (d < __builtin_huge_valf() && d > mx) mx = d;
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  const float hmax = red[0];
  __syncthreads();
  // g = smallest sqrt(H_kk) 2^-e_k over the live columns: what one unit of a column's integers
  // is worth relative to that column's own scale
  float gmin = __builtin_huge_valf();
  for (int64_t k = threadIdx.x; k < npad; k += 256) {
    int e = 0;
    if (k < n && hmax > 0.f) {
      const float d = Hdiag[k];
      if (d > 0.f && d < __builtin_huge_valf()) {
        const float t = (float)EMAX + rintf(0.5f * log2f(d / hmax));
        e = t < 0.f ? 0 : (t > (float)EMAX ? EMAX : (int)t);
        gmin = fminf(gmin, sqrtf(d) / (float)(1 << e));
      }
    }
    Cs[k] = (uint8_t)(1 << e);
  }
  red[threadIdx.x] = gmin;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fminf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  gmin = red[0];
  for (int t = threadIdx.x; t < mtiles; t += 256) Ptile[t] = 0;
  if (threadIdx.x == 0) {
    scale[0] = 1.f;
    scale[1] = 1.f;     // the fold applies the row factors; nothing is left for the solve
    scale[2] = hmax;
    // columns more than 2^18 below the largest one are held to its absolute precision only
    const float gfloor = ldexpf(sqrtf(hmax), -18);
    scale[3] = (gmin < __builtin_huge_valf() && gmin > gfloor) ? gmin : gfloor;
  }
}

// Flags of a tile of TM rows: some row needs three digits; some row's two-digit (three-digit)
// integers could overflow an int32 when summed over a whole row, so the digits cannot share
// one accumulator.
constexpr int TF_THREE = 1, TF_SUM2 = 2, TF_SUM3 = 4, TF_FOUR = 8;
__device__ __host__ inline int tile_digits(int flags) {
  return (flags & TF_FOUR) ? 4 : (flags & TF_THREE) ? 3 : 2;
}
__device__ __host__ inline bool tile_shared_acc(int flags) {
  if (flags & TF_FOUR) return false;
  return (flags & ((flags & TF_THREE) ? TF_SUM3 : TF_SUM2)) == 0;
}

// Row j: the largest |H_jk| 2^-e_k over k != j (the update of later sweeps reads whole rows)
// gives the row exponents for two and for three digits; the row asks for three digits unless 16 of its largest scaled entry stay below
// sqrt(H_jj) g (a unit of its 16-bit integers is then at most 2^-19 sqrt(H_jj H_kk) for
// every live column k), and sum_k |H_jk| 2^s tells whether any subset sum of the row's integers
// (times their column factors) stays inside an int32.
__global__ __launch_bounds__(256) void t_rowscale_kernel(const float* __restrict__ H, int64_t n,
                                                         int64_t ldh, const float* __restrict__ scale,
                                                         const float* __restrict__ Hdiag,
                                                         const uint8_t* __restrict__ Cs,
                                                         int8_t* __restrict__ S2,
                                                         int8_t* __restrict__ S3,
                                                         int16_t* __restrict__ Sneed,
                                                         int* __restrict__ Ptile) {
  __shared__ float rmx[256], rsum[256];
  const int64_t j = blockIdx.x;
  float mx = 0.f, sum = 0.f;
  if (j < n) {
    for (int64_t k = threadIdx.x; k < n; k += 256) {
      if (k == j) continue;
      const float a = fabsf(H[j * ldh + k]);
      sum += a;
      mx = fmaxf(mx, a / (float)Cs[k]);
    }
  }
  rmx[threadIdx.x] = mx;
  rsum[threadIdx.x] = sum;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      rmx[threadIdx.x] = fmaxf(rmx[threadIdx.x], rmx[threadIdx.x + w]);
      rsum[threadIdx.x] += rsum[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  mx = rmx[0];
  sum = rsum[0];
  int s2 = 0, s3 = 0;
  int need = -30000;          // smallest two-digit exponent that is precise enough; none for an empty row
  if (mx > 0.f && mx < __builtin_huge_valf()) {
    s2 = 14 - ilogbf(mx);
    if (ldexpf(mx, s2) > V2MAX) --s2;
    s3 = 22 - ilogbf(mx);
    if (ldexpf(mx, s3) > V3MAX) --s3;
    s2 = s2 < -120 ? -120 : (s2 > 110 ? 110 : s2);
    s3 = s3 < -120 ? -120 : (s3 > 110 ? 110 : s3);     // four digits use s3 + 8
    // |sum_k v_jk 2^e_k [..]| <= 2^s sum_k |H_jk| + 2^(EMAX-1) n  must stay below 2^31
    const int t = (sum < __builtin_huge_valf()) ? 29 - ilogbf(sum) : -1000;   // sum 2^t < 2^30
    const float dj = Hdiag[j];
    const bool dok = dj > 0.f && dj < __builtin_huge_valf();
    const float yard = dok ? sqrtf(dj) * scale[3] : 0.f;
    const bool two = dok && mx * 16.f <= yard;      // a unit of 16-bit integers is small enough
    const bool three = dok && mx <= 16.f * yard;    // a unit of 24-bit integers is
    const int flags = (two ? 0 : TF_THREE) | (three ? 0 : TF_FOUR) | (s2 <= t ? 0 : TF_SUM2) |
                      (s3 <= t ? 0 : TF_SUM3);
    if (flags != 0) atomicOr(&Ptile[j / TM], flags);
    if (yard > 0.f) need = 18 - ilogbf(yard);       // 2^-s <= 2^-18 yard, the bound that `two` tests
  }
  S2[j] = (int8_t)s2;
  S3[j] = (int8_t)s3;
  Sneed[j] = (int16_t)need;
}

// Hs[digit][j][k], digit 0 the most significant one: whole rows, k != j (the diagonal entry is 0;
// it enters through D_i).  The GEMM of a full sweep visits k < j only: it reads the tiles left of
// the diagonal tile from Hs and the diagonal tile itself from Hd[digit][tile][j % TM][k % TM],
// which holds the same digits for k < j and zeros elsewhere.
__global__ __launch_bounds__(256) void t_split_kernel(const float* __restrict__ H, int64_t n,
                                                      int64_t ldh, int64_t npad,
                                                      const uint8_t* __restrict__ Cs,
                                                      const int8_t* __restrict__ S2,
                                                      const int8_t* __restrict__ S3,
                                                      const int* __restrict__ Ptile,
                                                      int8_t* __restrict__ Hs, int8_t* __restrict__ Hd,
                                                      float* __restrict__ Wj) {
  const int64_t j = blockIdx.y;                                   // row of H
  const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;      // column
  if (k >= npad) return;
  const int P = tile_digits(Ptile[j / TM]);
  const int sj = (j < n) ? ((P == 2) ? S2[j] : (P == 3) ? S3[j] : S3[j] + 8) : 0;
  if (k == 0) Wj[j] = ldexpf(1.f, -sj);
  int iv = 0;
  if (j < n && k < n && k != j) {
    const float lim = (P == 2) ? V2MAX : (P == 3) ? V3MAX : 256.f * V3MAX;
    float v = rintf(ldexpf(H[j * ldh + k], sj) / (float)Cs[k]);
    v = (v == v) ? fminf(fmaxf(v, -lim), lim) : 0.f;
    iv = (int)v;
  }
  int dgt[4] = {0, 0, 0, 0};            // most significant first, P of them
  {
    int rest = iv;
    for (int q = P - 1; q >= 0; --q) {
      const int d = (int)(int8_t)(rest & 0xff);
      dgt[q] = d;
      rest = (rest - d) >> 8;
    }
  }
  const int64_t o = j * npad + k, ps = npad * npad;
  for (int q = 0; q < P; ++q) Hs[q * ps + o] = (int8_t)dgt[q];
  if (k / TM == j / TM) {
    const int64_t od = ((j / TM) * TM + (j % TM)) * TM + (k % TM), pd = npad * TM;
    for (int q = 0; q < P; ++q) Hd[q * pd + od] = (int8_t)((k < j) ? dgt[q] : 0);
  }
}

// May later sweeps update A_i instead of summing it again?  An update adds and removes whole rows
// of the integer matrix, entries right of the diagonal included, while a sweep that sums visits
// each pair once, left of the diagonal: the two agree exactly only if the integers are symmetric,
// v_jk 2^(e_k - s_j) = v_kj 2^(e_j - s_k), i.e. s_j = s - e_j with one s for the whole matrix.  That
// choice is made here when it costs no precision - every tile at two digits, s the largest value
// that keeps every row inside 16 bits, and every row still as fine as the two-digit rule asks -
// and then the update is allowed; otherwise the per-row exponents stay and every sweep sums.
__global__ __launch_bounds__(1024) void t_symscale_kernel(const int* __restrict__ Ptile, int mtiles, int64_t n,
                                                          int allow, const uint8_t* __restrict__ Cs,
                                                          int8_t* __restrict__ S2,
                                                          const int16_t* __restrict__ Sneed,
                                                          int* __restrict__ Tstat) {
  __shared__ int red[1024];
  const int tid = threadIdx.x;
  int smin = 1 << 20;
  for (int64_t j = tid; j < n; j += 1024)
    if (Sneed[j] > -30000) smin = min(smin, (int)S2[j] + (31 - __builtin_clz((unsigned)Cs[j])));
  red[tid] = smin;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (tid < w) red[tid] = min(red[tid], red[tid + w]);
    __syncthreads();
  }
  smin = red[0];
  __syncthreads();
  int bad = 0;
  for (int t = tid; t < mtiles; t += 1024)
    if (Ptile[t] & (TF_THREE | TF_FOUR)) bad = 1;
  for (int64_t j = tid; j < n; j += 1024) {
    const int sj = smin - (31 - __builtin_clz((unsigned)Cs[j]));
    if (sj < (int)Sneed[j] || sj < -120 || sj > 110) bad = 1;
  }
  red[tid] = bad;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (tid < w) red[tid] |= red[tid + w];
    __syncthreads();
  }
  const int ok = (allow != 0 && red[0] == 0 && smin < (1 << 20)) ? 1 : 0;
  if (ok)
    for (int64_t j = tid; j < n; j += 1024) S2[j] = (int8_t)(smin - (31 - __builtin_clz((unsigned)Cs[j])));
  if (tid == 0) {
    Tstat[0] = 0;
    Tstat[1] = 0;
    Tstat[2] = 0;       // no state yet
    Tstat[3] = ok;
    Tstat[4] = 0;
  }
}

// Tstat: [0] largest number of changed indices in a row, [1] their total, [2] A-state valid,
// [3] updates allowed for this layer, [4] number of 64-column chunks of changed columns.  The same
// test in every kernel of a sweep: update when at most 1 / kDeltaInv of the indices changed.
constexpr int kDeltaInv = 24;
constexpr int kDeltaChunk = 32;
__device__ inline bool t_use_delta(const int* __restrict__ st, int64_t m, int64_t n, int fmax) {
  return st[2] != 0 && st[3] != 0 && st[0] <= fmax && (int64_t)st[1] * kDeltaInv <= m * n;
}

// Zero-padded copy of Q (Qp, one byte per index, read by the fold) and, for the one-hot
// staging of the GEMM, the byte offset of each index's entry inside the one-hot LDS tile (Qo):
// row (i mod RW) * C + code of TK bytes, 16-byte chunks XOR-permuted by (row >> 1) & 3.
// One thread takes 16 consecutive indices (npad is a multiple of 16): one 16-byte store of codes
// and two of offsets; the codes come in one 16-byte load where the row of Q allows it.
__global__ __launch_bounds__(256) void pad_q_kernel(const uint8_t* __restrict__ Q, int64_t m,
                                                    int64_t n, int64_t ldq, int64_t npad, int nbits,
                                                    int vec, uint8_t* __restrict__ Qp,
                                                    uint16_t* __restrict__ Qo) {
  const int64_t i = blockIdx.y;
  const int64_t k0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (k0 >= npad) return;
  const int C = 1 << nbits, RW = TN >> nbits;
  uint32_t w[4] = {0u, 0u, 0u, 0u};
  if (i < m) {
    if (vec && k0 + 16 <= n) {
      const uint4 v = *reinterpret_cast<const uint4*>(Q + i * ldq + k0);
      w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
#pragma unroll
      for (int t = 0; t < 16; ++t)
        if (k0 + t < n) w[t >> 2] |= (uint32_t)Q[i * ldq + k0 + t] << (8 * (t & 3));
    }
  }
  const uint32_t cm = (uint32_t)(C - 1) * 0x01010101u;
#pragma unroll
  for (int u = 0; u < 4; ++u) w[u] &= cm;
  *reinterpret_cast<uint4*>(Qp + i * npad + k0) = uint4{w[0], w[1], w[2], w[3]};
  const int rbase = (int)(i % RW) * C, kc = (int)((k0 & (TK - 1)) >> 4);
  uint32_t o[8];
#pragma unroll
  for (int t = 0; t < 16; t += 2) {
    uint32_t pk = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int code = (int)((w[(t + h) >> 2] >> (8 * ((t + h) & 3))) & 0xffu);
      const int nrow = rbase + code;
      pk |= (uint32_t)(nrow * TK + (((kc ^ (nrow >> 1)) & 3) << 4) + (t + h)) << (16 * h);
    }
    o[t >> 1] = pk;
  }
  uint4* dst = reinterpret_cast<uint4*>(Qo + i * npad + k0);
  dst[0] = uint4{o[0], o[1], o[2], o[3]};
  dst[1] = uint4{o[4], o[5], o[6], o[7]};
}

// ---- changed indices of a sweep ----
// Row i: the columns whose code differs between the previous padded copy of Q and the current one,
// in ascending order, as j | old << 16 | new << 20 (at most fmax are stored; Fcnt holds the true
// count).
__global__ __launch_bounds__(256) void t_flips_kernel(const uint8_t* __restrict__ Qn,
                                                      const uint8_t* __restrict__ Qo, int64_t npad,
                                                      int fmax, uint32_t* __restrict__ Flist,
                                                      int* __restrict__ Fcnt) {
  __shared__ int wcnt[4];
  const int64_t i = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int base = 0;
  // 16 columns per thread and round (npad is a multiple of 128, so a thread's 16 are all inside or
  // all outside the row); the order inside a round is thread, then column
  for (int64_t k0 = 0; k0 < npad; k0 += 4096) {
    const int64_t k = k0 + 16 * tid;
    uint4 qn = uint4{0u, 0u, 0u, 0u}, qo = uint4{0u, 0u, 0u, 0u};
    if (k < npad) {
      qn = *reinterpret_cast<const uint4*>(Qn + i * npad + k);
      qo = *reinterpret_cast<const uint4*>(Qo + i * npad + k);
    }
    const uint32_t wn[4] = {qn.x, qn.y, qn.z, qn.w}, wo[4] = {qo.x, qo.y, qo.z, qo.w};
    int mine = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t x = wn[w] ^ wo[w];
#pragma unroll
      for (int b = 0; b < 4; ++b) mine += ((x >> (8 * b)) & 0xffu) != 0u;
    }
    // exclusive prefix of `mine` over the workgroup
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off, 64);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wcnt[wave] = incl;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      woff += (v < wave) ? wcnt[v] : 0;
      total += wcnt[v];
    }
    int pos = base + woff + incl - mine;
    if (mine > 0) {
#pragma unroll
      for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t cn = (wn[w] >> (8 * b)) & 0xffu, co = (wo[w] >> (8 * b)) & 0xffu;
          if (cn != co) {
            if (pos < fmax) Flist[i * fmax + pos] = (uint32_t)(k + 4 * w + b) | (co << 16) | (cn << 20);
            ++pos;
          }
        }
    }
    base += total;
    __syncthreads();
  }
  if (tid == 0) Fcnt[i] = base;
}

// Cbase[i] = number of 32-column chunks of changed columns in rows before i (exclusive prefix sum
// over the rows, one workgroup), Tstat[4] = their total: one wavefront of the update kernel per
// chunk.  Also the largest count of a row and the total (Tstat[0], Tstat[1]), and the mark that a
// completed sweep has left a valid state (Tstat[2]; this kernel runs from the second sweep on).
__global__ __launch_bounds__(1024) void t_chunks_kernel(const int* __restrict__ Fcnt, int64_t m, int fmax,
                                                        int* __restrict__ Cbase, int* __restrict__ Tstat) {
  __shared__ int wsum[16], wmax[16], wtot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t per = (m + 1023) / 1024;
  const int64_t b = tid * per, e = (b + per < m) ? b + per : m;
  auto chunks = [&](int c) {
    if (c > fmax) c = fmax;         // such a sweep sums again anyway; keep the table in range
    return (c + kDeltaChunk - 1) / kDeltaChunk;
  };
  int s = 0, mx = 0, tot = 0;
  for (int64_t i = b; i < e; ++i) {
    const int c = Fcnt[i];
    s += chunks(c);
    mx = max(mx, c);
    tot += c;
  }
  // inclusive scan of s within the wavefront, then over the 16 wavefronts
  int incl = s;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    mx = max(mx, __shfl_xor(mx, o, 64));
    tot += __shfl_xor(tot, o, 64);
  }
  if (lane == 63) wsum[wave] = incl;
  if (lane == 0) {
    wmax[wave] = mx;
    wtot[wave] = tot;
  }
  __syncthreads();
  int before = 0, total = 0, gmax = 0, gtot = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int v = wsum[w];
    if (w < wave) before += v;
    total += v;
    gmax = max(gmax, wmax[w]);
    gtot += wtot[w];
  }
  if (tid == 0) {
    Tstat[0] = gmax;
    Tstat[1] = gtot;
    Tstat[2] = 1;
    Tstat[4] = total;
    Cbase[m] = total;
  }
  int run = before + incl - s;
  for (int64_t i = b; i < e; ++i) {
    Cbase[i] = run;
    run += chunks(Fcnt[i]);
  }
}

typedef int intx16 __attribute__((ext_vector_type(16)));

// 16 one-hot operand bytes: byte t of word w is cs (the column factor 2^e_k) where the code byte
// equals b, else 0.  Codes and b are below 16: 0x10 - (code ^ b) has bit 4 set exactly on a match.
__device__ inline int4v onehot16(uint4 q, uint32_t brep, uint4 cs) {
  auto one = [&](uint32_t qw, uint32_t cw) -> int {
    const uint32_t hit = (0x10101010u - (qw ^ brep)) & 0x10101010u;   // 0x10 per matching byte
    uint32_t msk = hit >> 4;                                          // 0x01
    msk |= msk << 1;
    msk |= msk << 2;
    msk |= msk << 4;                                                  // 0xff
    return (int)(cw & msk);
  };
  int4v r;
  r[0] = one(q.x, cs.x);
  r[1] = one(q.y, cs.y);
  r[2] = one(q.z, cs.z);
  r[3] = one(q.w, cs.w);
  return r;
}

// ---- update of A_i for the changed columns of a sweep ----
// One wavefront per chunk of 32 changed columns j of a row i (rows differ widely in how many of
// their indices still change, so the unit of work is the chunk, not the row): one MFMA row tile of
// 32 gathered rows of Hs; the 32 columns of the product are the 16 old codes and the 16 new codes
// (one-hot operands built in registers from the two padded copies of Q), each digit of H in its own
// int32 accumulator:  Z[j, c] = sum_k v_jk 2^e_k [code_k == c]  exactly.  Then, with d_j = e_new(j) -
// e_old(j) and w_j = 2^-s_j, the chunk's share of
//   A[a, b] += sum_j d_j[a] w_j Znew[j, b] + sum_j d_j[b] w_j Zold[j, a]
// is accumulated per lane in float64 (a lane owns one column of Z, i.e. one b or one a) and written
// to the chunk's slot of Dpart; the solve kernel adds a row's slots to its state in a fixed order.
// The kernel is bound by the gathered loads.  They are issued as whole 128-byte lines (8 lanes per
// row, 8 rows per instruction) - a request per row and k-step in the operand layout (2 lanes per
// row) costs the cache four look-ups per line - and turned into the operand layout through a
// wavefront-private piece of LDS (rows padded to 144 bytes: conflict-free 16-byte reads of 16
// consecutive rows); the next batch's lines are requested before the current batch is multiplied.
constexpr int DROWB = 144;                       // LDS bytes per staged row
constexpr int DSTAGE = 2 * 32 * DROWB;           // per wavefront: two digits x 32 rows
template <int NBITS>
__global__ __launch_bounds__(256, 3) void t_delta_kernel(const int8_t* __restrict__ Hs, int64_t npad,
                                                         const uint8_t* __restrict__ Qnew,
                                                         const uint8_t* __restrict__ Qold,
                                                         const uint8_t* __restrict__ Cs,
                                                         const float* __restrict__ Wj,
                                                         const uint32_t* __restrict__ Flist,
                                                         const int* __restrict__ Fcnt,
                                                         const int* __restrict__ Cbase,
                                                         const int* __restrict__ Tstat, int fmax,
                                                         int64_t m, int64_t n,
                                                         double* __restrict__ Dpart) {
  constexpr int C = 1 << NBITS;
  __shared__ __attribute__((aligned(16))) unsigned char dsm[4][DSTAGE];
  if (!t_use_delta(Tstat, m, n, fmax)) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = (int)blockIdx.x * 4 + wave;      // chunk number
  if (q >= Tstat[4]) return;
  // row of this chunk: the last i with Cbase[i] <= q (Cbase is non-decreasing, Cbase[m] = total)
  int lo = 0, hi = (int)m;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (Cbase[mid] <= q) lo = mid; else hi = mid;
  }
  const int64_t i = lo;
  const int t0 = (q - Cbase[lo]) * kDeltaChunk;
  const int cnt = Fcnt[i];
  const int c = lane & 31, kh = lane >> 5;
  const uint32_t brep = 0x01010101u * (uint32_t)(c & 15);
  const uint8_t* __restrict__ qrow = ((c < 16) ? Qold : Qnew) + i * npad + 16 * kh;
  const uint8_t* __restrict__ csrow = Cs + 16 * kh;
  const int64_t ps = npad * npad;

  // lane c (and c + 32) holds entry c of the chunk: changed column, old and new code, row factor
  const int e0 = t0 + c;
  const uint32_t ent = (e0 < cnt) ? Flist[i * fmax + e0] : 0u;
  const int64_t jrow = ent & 0xffffu;
  const float wrow = (e0 < cnt) ? Wj[jrow] : 0.f;       // entries beyond the count add nothing
  // gather side: instruction t fetches rows 8 t + lane / 8, 16-byte piece lane % 8 of the line
  const int gr = lane >> 3, gp = lane & 7;
  const int8_t* __restrict__ grow[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int64_t jt = __shfl((int)jrow, 8 * t + gr, 64);
    grow[t] = Hs + jt * npad + 16 * gp;
  }
  unsigned char* __restrict__ stage = dsm[wave];
  const int wr_off = gr * DROWB + gp * 16;               // + (8 t) * DROWB + digit * 32 * DROWB
  const int rd_off = c * DROWB + kh * 16;                // + 32 * step + digit * 32 * DROWB

  intx16 acc[2];
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[d][v] = 0;
  int4v g[4][2];
  uint4 q16[4], cs16[4];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int d = 0; d < 2; ++d) g[t][d] = *reinterpret_cast<const int4v*>(grow[t] + d * ps + k0);
      q16[t] = *reinterpret_cast<const uint4*>(qrow + k0 + 32 * t);
      cs16[t] = *reinterpret_cast<const uint4*>(csrow + k0 + 32 * t);
    }
  };
  fetch(0);
  for (int64_t k0 = 0; k0 < npad; k0 += 128) {
    // the lines of this batch into LDS (only this wavefront touches its stage, and its LDS
    // operations execute in order), the one-hot operands of the batch, then the next batch's loads
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int d = 0; d < 2; ++d)
        *reinterpret_cast<int4v*>(stage + d * 32 * DROWB + 8 * t * DROWB + wr_off) = g[t][d];
    int4v bf[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) bf[t] = onehot16(q16[t], brep, cs16[t]);
    if (k0 + 128 < npad) fetch(k0 + 128);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        const int4v a = *reinterpret_cast<const int4v*>(stage + d * 32 * DROWB + rd_off + 32 * t);
        acc[d] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bf[t], acc[d], 0, 0, 0);
      }
    }
  }
  // fold: row r of the tile sits in register v = 4 (r / 8) + r % 4 of the lanes with kh = (r / 4) % 2
  double R[C];
#pragma unroll
  for (int a2 = 0; a2 < C; ++a2) R[a2] = 0.0;
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    const int v = 4 * (r >> 3) + (r & 3), khr = (r >> 2) & 1;
    const uint32_t er = (uint32_t)__builtin_amdgcn_readlane((int)ent, r);
    const float wr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wrow), r));
    const double z = (double)acc[0][v] * 256.0 + (double)acc[1][v];
    const double x = (kh == khr) ? (double)wr * z : 0.0;
    const int ao = (int)((er >> 16) & 15u), an = (int)((er >> 20) & 15u);
#pragma unroll
    for (int a2 = 0; a2 < C; ++a2) {
      const double f = (double)((an == a2) - (ao == a2));     // scalar: -1, 0 or 1
      R[a2] = fma(f, x, R[a2]);
    }
  }
  // the chunk's A[a, b]: R of the lanes that own column "new b", element a, plus R of the lanes
  // that own column "old a", element b (two lanes each: kh = 0, 1); through the same piece of LDS
  double* __restrict__ Rs = reinterpret_cast<double*>(stage);        // [lane][C], 8 KB at most
#pragma unroll
  for (int a2 = 0; a2 < C; ++a2) Rs[lane * C + a2] = R[a2];
  __builtin_amdgcn_wave_barrier();
  for (int e = lane; e < C * C; e += 64) {
    const int a2 = e / C, b2 = e % C;
    Dpart[(int64_t)q * C * C + e] =
        (Rs[(16 + b2) * C + a2] + Rs[(48 + b2) * C + a2]) + (Rs[a2 * C + b2] + Rs[(32 + a2) * C + b2]);
  }
}

// ---- the GEMM with fold epilogue ----
// LDS: T_S stages of { A tile: TM rows x 64 bytes (one digit of 64 k), one-hot B tile: TN rows
// x 64 bytes }.  A tiles arrive by direct-to-LDS buffer loads; such a load writes 64 x 16
// consecutive bytes, so rows cannot be padded and the 16-byte chunks of a row are stored in
// XOR-permuted order instead (chunk c of row r at c ^ ((r >> 1) & 3), both tiles).
// The one-hot tile is never rebuilt: it starts as zeros and each thread owns a fixed set of
// (row i, k) positions whose single entry it moves - it clears the one it wrote when the stage
// was last used and sets the new one (in-order LDS writes of one thread).
constexpr int T_S = 3;
constexpr int T_ROWB = TK;
constexpr int T_ATILEB = TM * T_ROWB;
constexpr int T_BTILEB = TN * T_ROWB;
constexpr int T_STAGEB = T_ATILEB + T_BTILEB;
constexpr int T_LDS_BYTES = T_S * T_STAGEB;

template <int V> struct IntC { static constexpr int value = V; };

// Workgroup = (slab of RW rows i, group g of row tiles {g, mtiles - 1 - g} of H): every
// workgroup runs the same number of k-steps per digit.  Three LDS stages and one barrier per
// k-step: the barrier at the top of step k publishes the data of step k + 1 and frees the
// stage of step k - 1, which is refilled for step k + 2; the first MFMA fragments of step
// k + 1 are read during step k, so no wavefront starts a step waiting for LDS.
//
// The fold  M_i[a, b] += [Q_ij == a] 2^-s_j Z[j, (i, b)]  is an outer product per row j, and
// v_mfma_f32_16x16x1_4b_f32 computes four independent 16 x 16 outer products per
// instruction, one per group of 16 lanes.  In the 32 x 32 accumulator tile lane l holds
// column l % 32 and register v holds one row j per lane half, so the 16-lane groups are
// (lane half, 16-column half) and register v itself (converted to float) is the right
// operand; the left operand is 2^-s_j where the code of (this lane's row i, that j) equals
// l % C, else 0.  With C < 16 a 16-column group spans several rows i and only the diagonal
// C x C blocks of the 16 x 16 result are meaningful; the others are never stored.
template <int NBITS>
__global__ __launch_bounds__(64 * TNW, 2) void t_accum_kernel(const int8_t* __restrict__ Hs,
                                                           const int8_t* __restrict__ Hd,
                                                           const int* __restrict__ Tstat, int fmax,
                                                           int64_t m_rows, int64_t n_cols,
                                                           int64_t npad, const uint8_t* __restrict__ Qp,
                                                           const uint16_t* __restrict__ Qo,
                                                           const uint8_t* __restrict__ Cs,
                                                           const float* __restrict__ Wj,
                                                           const int* __restrict__ Ptile,
                                                           int64_t mpad, int mtiles, int ngroups,
                                                           float* __restrict__ Apart) {
  // a sweep that updates A_i from the changed columns does not sum it again
  if (t_use_delta(Tstat, m_rows, n_cols, fmax)) return;
  constexpr int C = 1 << NBITS;
  constexpr int RW = TN >> NBITS;             // rows i per workgroup
  constexpr int EPT = (RW * TK) / (64 * TNW); // one-hot positions per thread and stage
  constexpr int EW = EPT / 2;                 // dwords of offsets per thread and stage
  constexpr int CW = EPT / 4;                 // dwords of one-hot values per thread and stage
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

  // Workgroups are dealt to the 8 XCDs round-robin by flat index; items are ordered
  // (group, slab) and each XCD takes a contiguous eighth, so the workgroups sharing an L2
  // read the same rows of H.
  const int nslabs = (int)(mpad / RW);
  const int64_t total = (int64_t)nslabs * ngroups;
  const int64_t per = (total + 7) / 8;
  const int64_t qq = blockIdx.x >> 3;
  const int64_t item = (int64_t)(blockIdx.x & 7) * per + qq;
  if (qq >= per || item >= total) return;
  const int group = (int)(item / nslabs);
  const int64_t i0 = (item % nslabs) * RW;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kh = lane >> 5, l32 = lane & 31;

  for (int e = tid; e < T_LDS_BYTES / 16; e += 64 * TNW)
    reinterpret_cast<uint4*>(smem)[e] = uint4{0u, 0u, 0u, 0u};

  // one-hot staging: this thread owns row il and the EPT consecutive k from kk0 of every
  // stage.  q3..q0 hold the packed tile offsets of the last three scattered steps and of the
  // next one; the stage written for step s held step s - 3 (stages rotate over all steps of
  // the workgroup, across digits and row tiles), so its entries are cleared with q3.  Before
  // the first steps the "old" positions are this thread's own code-0 positions (zeros already).
  // With few bits per index a thread owns many positions and that queue would not fit the
  // register file: the wavefront then zeroes its part of the tile with full-width stores
  // instead (the rows (il, code) of its threads are 64 consecutive rows of the tile, 4 KB that
  // no other wavefront writes, and the LDS operations of one wavefront execute in order).
  constexpr bool QUEUE = NBITS >= 3;
  constexpr int QW = QUEUE ? EW : 1;
  const int ex_il = (tid * EPT) / TK, ex_kk0 = (tid * EPT) % TK;
  const uint32_t* __restrict__ qorow = reinterpret_cast<const uint32_t*>(Qo + (i0 + ex_il) * npad + ex_kk0);
  const uint32_t* __restrict__ csrow = reinterpret_cast<const uint32_t*>(Cs + ex_kk0);
  uint32_t q3[QW], q2[QW], q1[QW], q0[EW], cv[CW];
  if constexpr (QUEUE) {
#pragma unroll
    for (int w = 0; w < EW; ++w) {
      uint32_t pk = 0;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int nrow = ex_il * C, kk = ex_kk0 + 2 * w + h;
        pk |= (uint32_t)(nrow * T_ROWB + ((((kk >> 4) ^ (nrow >> 1)) & 3) << 4) + (kk & 15)) << (16 * h);
      }
      q3[w] = q2[w] = q1[w] = pk;
    }
  }

  // direct load of the A tile: one instruction covers 16 rows x 64 bytes; TM / 16 of them are
  // dealt to the wavefronts
  constexpr int ALD = (TM / 16) / TNW;
  const int dr = lane >> 2;
  const int dc = (lane & 3) ^ ((dr >> 1) & 3);
  uint32_t voff[ALD], voffd[ALD];      // in a row tile of Hs (row stride npad) and in a diagonal tile of Hd (TM)
#pragma unroll
  for (int a = 0; a < ALD; ++a) {
    voff[a] = (uint32_t)((int64_t)((wave + TNW * a) * 16 + dr) * npad + dc * 16);
    voffd[a] = (uint32_t)(((wave + TNW * a) * 16 + dr) * TM + dc * 16);
  }

  const int rswz = (l32 >> 1) & 3;
  // per-lane LDS byte offsets of the fragments inside a stage
  const int aoff = l32 * T_ROWB;
  const int boff = T_ATILEB + (wave * 64 + l32) * T_ROWB;
  int st = 0;                // stage of the next k-step; rotates over all steps of the workgroup
  __syncthreads();

  for (int half = 0; half < 2; ++half) {
    const int mt = (half == 0) ? group : mtiles - 1 - group;
    if (half == 1 && mt == group) break;
    const int64_t jt0 = (int64_t)mt * TM;
    const int nk = (int)((jt0 + TM) / TK);    // tiles right of the diagonal are never needed (nk >= 2)
    const int tflags = __builtin_amdgcn_readfirstlane(Ptile[mt]);
    const int P = tile_digits(tflags);
    const bool shared_acc = tile_shared_acc(tflags);   // the digits may share the accumulators

    auto load_q = [&](int k) {
#pragma unroll
      for (int w = 0; w < EW; ++w) q0[w] = qorow[(k * TK) / 2 + w];
#pragma unroll
      for (int w = 0; w < CW; ++w) cv[w] = csrow[(k * TK) / 4 + w];
    };
    // clear the entries of the step that used this stage last (q3, or the whole part of this
    // wavefront), set those of q0, rotate
    auto scatter = [&](int st) {
      unsigned char* Bs = smem + st * T_STAGEB + T_ATILEB;
      if constexpr (QUEUE) {
#pragma unroll
        for (int w = 0; w < EW; ++w) {
          Bs[q3[w] & 0xffffu] = 0;
          Bs[q3[w] >> 16] = 0;
        }
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          *reinterpret_cast<uint4*>(Bs + wave * 4096 + t * 1024 + lane * 16) = uint4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int w = 0; w < EW; ++w) {
        Bs[q0[w] & 0xffffu] = (unsigned char)((cv[w >> 1] >> (16 * (w & 1))) & 0xffu);
        Bs[q0[w] >> 16] = (unsigned char)((cv[w >> 1] >> (16 * (w & 1) + 8)) & 0xffu);
        if constexpr (QUEUE) {
          q3[w] = q2[w];
          q2[w] = q1[w];
          q1[w] = q0[w];
        }
      }
    };

    intx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0;

    struct Frags {
      int4v a[4], b[2];
    };
    auto load_frags = [&](Frags& f, int st, int ks) {
      const unsigned char* S0 = smem + st * T_STAGEB;
      const int cs = ((2 * ks + kh) ^ rswz) << 4;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        f.a[i] = *reinterpret_cast<const int4v*>(S0 + aoff + i * 32 * T_ROWB + cs);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
        f.b[jn] = *reinterpret_cast<const int4v*>(S0 + boff + jn * 32 * T_ROWB + cs);
    };
    auto mma = [&](const Frags& f) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.a[i], f.b[jn], acc[i][jn], 0, 0, 0);
    };

    const int acmp = lane & (C - 1);

    for (int dg = 0; dg < P; ++dg) {
      int4v rsA, rsD;
      {
        const uint64_t ad = (uint64_t)(uintptr_t)(Hs + ((int64_t)dg * npad + jt0) * npad);
        rsA[0] = (int)(uint32_t)ad;
        rsA[1] = (int)(uint32_t)((ad >> 32) & 0xffffu);
        rsA[2] = (int)(uint32_t)((int64_t)TM * npad);
        rsA[3] = 0x00020000;
        const uint64_t dd = (uint64_t)(uintptr_t)(Hd + ((int64_t)dg * npad + jt0) * TM);
        rsD[0] = (int)(uint32_t)dd;
        rsD[1] = (int)(uint32_t)((dd >> 32) & 0xffffu);
        rsD[2] = (int)(uint32_t)(TM * TM);
        rsD[3] = 0x00020000;
      }
      // the last two k-steps are the diagonal tile, whose copy in Hd is zero for k >= j
      auto issue = [&](int k, int st) {
        if (k < nk - TM / TK) {
#pragma unroll
          for (int a = 0; a < ALD; ++a)
            load16_to_lds(rsA, lds0 + st * T_STAGEB + (wave + TNW * a) * 1024, voff[a], (uint32_t)k * (uint32_t)TK);
        } else {
#pragma unroll
          for (int a = 0; a < ALD; ++a)
            load16_to_lds(rsD, lds0 + st * T_STAGEB + (wave + TNW * a) * 1024, voffd[a],
                          (uint32_t)(k - (nk - TM / TK)) * (uint32_t)TK);
        }
      };
      if (dg > 0 && shared_acc) {
        // next digit: everything so far moves up by one digit
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] <<= 8;
      }

      // every stage is free here (start of the kernel, or the barrier after the previous pass)
      {
        const int st1 = (st == 2) ? 0 : st + 1;
        load_q(0);
        issue(0, st);
        issue(1, st1);
        scatter(st);
        load_q(1);
        scatter(st1);
        load_q(nk > 2 ? 2 : nk - 1);
      }
      wait_all_loads();
      __syncthreads();
      Frags f0, f1;
      load_frags(f0, st, 0);   // step 0 repeats the barrier, which costs nothing here

      // One k-step.  PRODUCE: stage the operands of step k + 2 (the Q offsets of step k + 3
      // are fetched with a clamped index so that the load is unconditional).  PREFETCH: read
      // the first fragments of step k + 1.
      auto step = [&](int k, auto PRODUCE, auto PREFETCH) {
        const int st1 = (st == 2) ? 0 : st + 1, st2 = (st == 0) ? 2 : st - 1;
        wait_all_loads();
        __syncthreads();
        if constexpr (decltype(PRODUCE)::value != 0) {
          scatter(st2);
          load_q(k + 3 < nk ? k + 3 : nk - 1);
          issue(k + 2, st2);
        }
        load_frags(f1, st, 1);
        mma(f0);
        if constexpr (decltype(PREFETCH)::value != 0) load_frags(f0, st1, 0);
        mma(f1);
        st = st1;
      };
#pragma unroll 1
      for (int k = 0; k < nk - 2; ++k) step(k, IntC<1>{}, IntC<1>{});
      step(nk - 2, IntC<0>{}, IntC<1>{});
      step(nk - 1, IntC<0>{}, IntC<0>{});
      // the LDS stages are reused by the next pass; slower wavefronts may still be reading
      __syncthreads();
      if (shared_acc && dg + 1 < P) continue;

      // fold: register v of tile (i, jn) is row j = i*32 + (v>>2)*8 + kh*4 + (v&3) of the tile.
      // D[jn] = four 16 x 16 blocks (lane half, column half) of column tile jn.  Accumulators
      // that hold a single digit are folded with that digit's weight and start again from 0.
      const float dgw = shared_acc ? 1.f : ldexpf(1.f, 8 * (P - 1 - dg));
      const bool first_fold = half == 0 && (shared_acc || dg == 0);   // nothing stored yet
      floatx16 D[2];
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int v = 0; v < 16; ++v) D[jn][v] = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint32_t qd[2][4];
        float4 wj[4];
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
          const int il = (wave * 64 + jn * 32 + l32) >> NBITS;
          const uint8_t* __restrict__ qr = Qp + (i0 + il) * npad + jt0 + i * 32 + kh * 4;
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) qd[jn][vq] = *reinterpret_cast<const uint32_t*>(qr + vq * 8);
        }
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          wj[vq] = *reinterpret_cast<const float4*>(Wj + jt0 + i * 32 + kh * 4 + vq * 8);
          wj[vq].x *= dgw;
          wj[vq].y *= dgw;
          wj[vq].z *= dgw;
          wj[vq].w *= dgw;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float4 w4 = wj[v >> 2];
          const float wv = (v & 3) == 0 ? w4.x : (v & 3) == 1 ? w4.y : (v & 3) == 2 ? w4.z : w4.w;
#pragma unroll
          for (int jn = 0; jn < 2; ++jn) {
            const int code = (int)((qd[jn][v >> 2] >> (8 * (v & 3))) & 0xffu);
            const float sel = (code == acmp) ? wv : 0.f;
            D[jn] = __builtin_amdgcn_mfma_f32_16x16x1f32(sel, (float)acc[i][jn][v], D[jn], 0, 0, 0);
            acc[i][jn][v] = 0;
          }
        }
      }
      // D[jn][4 B + r] = block B = 2 * (lane half of the source) + (16-column half), element
      // (row 4 (lane / 16) + r, column lane % 16): rows are (i', a), columns (i'', b) within the
      // 16-column group; keep i' == i'' and add the two lane halves.  Later folds add to what this
      // same thread stored after the first.
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int ch = 0; ch < 2; ++ch)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int mrow = 4 * (lane >> 4) + r, ncol = lane & 15;
            if ((mrow >> NBITS) != (ncol >> NBITS)) continue;
            float v = D[jn][4 * ch + r] + D[jn][4 * (2 + ch) + r];
            const int col = wave * 64 + jn * 32 + ch * 16 + ncol;      // (row i, code b) pair of the slab
            const int il = col >> NBITS, bb = col & (C - 1), aa = mrow & (C - 1);
            float* dst = Apart + ((int64_t)group * mpad + i0 + il) * C * C + aa * C + bb;
            if (!first_fold) v += *dst;
            *dst = v;
          }
    }
  }
}

// ---- per-row assembly and solve (one wavefront per row, float64) ----
__global__ __launch_bounds__(64) void t_solve_kernel(const float* __restrict__ Apart, int ngroups,
                                                     const int* __restrict__ Tstat, int fmax, int64_t m_rows,
                                                     double* __restrict__ Astate, int* __restrict__ Tlog,
                                                     const int* __restrict__ Cbase,
                                                     const double* __restrict__ Dpart,
                                                     double* __restrict__ Vstate, int* __restrict__ Nstate,
                                                     const uint32_t* __restrict__ Flist,
                                                     const int* __restrict__ Fcnt,
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
  __shared__ float binD[16][65], binB[16][65];      // 65: the 16 codes' partials fall into 16 banks
  __shared__ int binC[16][65];
  for (int a = 0; a < C; ++a) {
    binD[a][tid] = 0.f;
    binB[a][tid] = 0.f;
    binC[a][tid] = 0;
  }
  // After a sweep that brought S_i H0 S_i^T up to date from the changed columns, the per-code sums
  // of the row (diagonal of H, G, counts) are brought up to date the same way: the state of the
  // sweep before plus the signed contributions of the changed columns, instead of a pass over
  // the whole row of G and Q.
  const bool from_state = t_use_delta(Tstat, m_rows, n, fmax);
  if (Tlog != nullptr && i == 0 && tid == 0) {
    Tlog[0] = from_state ? 1 : 0;
    Tlog[1] = Tstat[0];
    Tlog[2] = Tstat[1];
  }
  if (!from_state) {
    // 16 columns per lane are fetched before the first is binned: the row of G comes from HBM,
    // and one column at a time would pay that latency n / 64 times over
    for (int64_t j0 = 0; j0 < n; j0 += 64 * 16) {
      int qa[16];
      float hv[16], gv[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int64_t j = j0 + tid + 64 * u;
        const int64_t jc = (j < n) ? j : n - 1;       // clamped: the loads stay unconditional
        const int qv = Q[i * ldq + jc];
        qa[u] = (j < n) ? (qv & (C - 1)) : -1;
        hv[u] = Hdiag[jc];
        gv[u] = G[i * ldg + jc];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int a = qa[u];
        if (a >= 0) {
          binD[a][tid] += hv[u];     // lane-private bins: plain read-modify-write
          binB[a][tid] += gv[u];
          binC[a][tid] += 1;
        }
      }
    }
  } else {
    // changed columns of this row: j | old code << 16 | new code << 20 (at most fmax of them, or
    // the sweep would not have been updated)
    const int nf = Fcnt[i];
    const uint32_t* __restrict__ fl = Flist + (int64_t)i * fmax;
    // four list entries per lane are fetched together, then their eight gathered values: two
    // round trips to memory per 256 changed columns
    for (int f0 = 0; f0 < nf; f0 += 256) {
      uint32_t ev[4];
      float hv[4], gv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int f = f0 + tid + 64 * u;
        ev[u] = fl[f < nf ? f : 0];                 // clamped: the loads stay unconditional
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t j = ev[u] & 0xffffu;
        hv[u] = Hdiag[j];
        gv[u] = G[i * ldg + j];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (f0 + tid + 64 * u < nf) {
          const int co = (ev[u] >> 16) & 15, cn = (ev[u] >> 20) & 15;
          binD[co][tid] -= hv[u];
          binB[co][tid] -= gv[u];
          binC[co][tid] -= 1;
          binD[cn][tid] += hv[u];
          binB[cn][tid] += gv[u];
          binC[cn][tid] += 1;
        }
      }
    }
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
    if (from_state) {
      sd += Vstate[(i * 2 + 0) * C + tid];
      sb += Vstate[(i * 2 + 1) * C + tid];
      c0 += Nstate[i * C + tid];
    }
    if (Vstate != nullptr) {
      Vstate[(i * 2 + 0) * C + tid] = sd;
      Vstate[(i * 2 + 1) * C + tid] = sb;
      Nstate[i * C + tid] = c0;
    }
    Dg[tid] = sd;
    rhs[tid] = sb;
    cnt[tid] = c0;
    dead[tid] = (c0 == 0);
  }
  __syncthreads();
  // Off-diagonal part S_i H0 S_i^T: after a sweep that summed it, M + M^T with M the sum of the
  // per-group partial folds (coalesced reads), which also becomes the state that later sweeps
  // update; after a sweep that updated it, the state itself.
  __shared__ double Ms[16][17];
  if (!from_state) {
    const int64_t gs = mpad * C * C;
    // all loads of up to 16 groups x 4 entries are issued before the first is used: one round
    // trip to memory instead of one per four groups
    const float* __restrict__ P0 = Apart + i * C * C + tid;
    double sacc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int g0 = 0; g0 < ngroups; g0 += 16) {
      float v[4][16];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int g = 0; g < 16; ++g)
        {
          // clamped address, value discarded when out of range: the loads stay unconditional
          const bool ok = tid + 64 * u < C * C && g0 + g < ngroups;
          const float t = P0[(ok ? 64 * u : -tid) + (int64_t)(ok ? g0 + g : 0) * gs];
          v[u][g] = ok ? t : 0.f;
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        // fixed order: four interleaved running sums over the groups, as ((s0 + s1) + (s2 + s3))
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (int g = 0; g < 16; g += 4) {
          s0 += (double)v[u][g];
          s1 += (double)v[u][g + 1];
          s2 += (double)v[u][g + 2];
          s3 += (double)v[u][g + 3];
        }
        sacc[u] += (s0 + s1) + (s2 + s3);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = tid + 64 * u;
      if (e < C * C) Ms[e / C][e % C] = sacc[u];
    }
  }
  __syncthreads();
  if (from_state) {
    // the state of the sweep before plus this sweep's chunks of changed columns, added in the
    // order of the chunks; the loads of four chunks and of this thread's (up to) four entries
    // are issued together, so a row costs one round trip to memory per four chunks
    const int c0 = Cbase[i], c1 = Cbase[i + 1];
    const int64_t CC = (int64_t)C * C;
    double vv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = tid + 64 * u;
      vv[u] = Astate[i * CC + (e < CC ? e : 0)];
    }
    for (int cc = c0; cc < c1; cc += 4) {
      double t[4][4];
#pragma unroll
      for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = tid + 64 * u;
          const bool ok = cc + w < c1 && e < CC;          // clamped address, value discarded
          const double x = Dpart[(int64_t)(ok ? cc + w : c0) * CC + (ok ? e : 0)];
          t[w][u] = ok ? x : 0.0;
        }
#pragma unroll
      for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int u = 0; u < 4; ++u) vv[u] += t[w][u];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = tid + 64 * u;
      if (e < CC) {
        if (c1 > c0) Astate[i * CC + e] = vv[u];
        const int a = e / C, b = e % C;
        double v = vv[u];
        if (a == b) { v += Dg[a]; diag0[a] = v; }
        A[a][b] = v;
      }
    }
  } else {
    for (int e = tid; e < C * C; e += 64) {
      const int a = e / C, b = e % C;
      double v = Ms[a][b] + Ms[b][a];
      Astate[i * C * C + e] = v;
      if (a == b) { v += Dg[a]; diag0[a] = v; }
      A[a][b] = v;
    }
  }
  __syncthreads();
  // Cholesky of the non-empty principal submatrix and the two triangular solves, in registers:
  // lane r < C holds row r of the lower triangle; a value of another lane comes by v_readlane
  // (the lane index is a compile-time constant in the unrolled loops), so the column-to-column
  // chain has no LDS round trip and no barrier.  A code whose column is empty (count 0) or
  // numerically dependent (pivot <= 1e-10 of its original diagonal, or not finite) is dropped:
  // unit pivot, zero column, zero right-hand side.
  auto bcast = [](double v, int src) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)u, src);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), src);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
  };
  const bool act = tid < C;
  double a[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) a[c] = (act && c <= tid) ? A[tid][c] : 0.0;
  int dd = act ? dead[tid] : 1;
  const double d0 = act ? diag0[tid] : 1.0;
  double s = (act && !dd) ? rhs[tid] : 0.0;
  double mydiag = 1.0;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    if (k < C) {
      const double piv = bcast(a[k], k);
      int dk = __builtin_amdgcn_readlane(dd, k);
      const double d0k = bcast(d0, k);
      if (!dk && (!(piv > 1e-10 * d0k) || !(piv < 1.79e308))) dk = 2;
      const double dkk = dk ? 1.0 : sqrt(piv);
      if (tid == k) {
        dd = dk;
        mydiag = dkk;
      }
      const double l = (tid > k && !dk && !dd) ? a[k] / dkk : 0.0;     // L[r][k]
      a[k] = (tid == k) ? dkk : l;
      if (!dk) {
#pragma unroll
        for (int c = k + 1; c < 16; ++c)
          if (c < C) a[c] -= l * bcast(l, c);       // used for c <= r only
      }
    }
  }
  // a pivot dropped after this lane's right-hand side was taken
  if (dd) s = 0.0;
  const double rd = (act && !dd) ? 1.0 / mydiag : 0.0;
  // forward: y_k = s_k / L_kk, then s_r -= L[r][k] y_k for r > k
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    if (k < C) {
      const double yk = bcast(s * rd, k);
      if (tid == k) s = yk;
      if (tid > k) s -= a[k] * yk;
    }
  }
  // backward with L^T: lane r needs L[k][r], k > r, i.e. column r: through LDS once
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 16; ++c)
    if (act && c <= tid) A[tid][c] = a[c];
  __syncthreads();
  double col[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) col[k] = (act && k > tid && k < C) ? A[k][tid] : 0.0;
#pragma unroll
  for (int k = 15; k >= 0; --k) {
    if (k < C) {
      const double xk = bcast(s * rd, k);
      if (tid == k) s = xk;
      if (tid < k) s -= col[k] * xk;
    }
  }
  if (act) {
    if (dd) {
      if (empty_mode == GANQ_EMPTY_ZERO || dd == 2) T[i * C + tid] = 0.f;
    } else {
      T[i * C + tid] = (float)s;
    }
  }
  if (empty_count != nullptr) {
    const unsigned long long dm = __builtin_amdgcn_ballot_w64(act && dd != 0);
    if (tid == 0) empty_count[i] = __builtin_popcountll(dm);
  }
}

inline int64_t t_npad(int64_t n) { return ceil_div(n, TM) * TM; }
inline int64_t t_mpad(int64_t m, int nbits) { const int64_t rw = TN >> nbits; return ceil_div(m, rw) * rw; }
inline int t_groups(int64_t n) { return (int)((ceil_div(n, TM) + 1) / 2); }

struct TScratch {
  float* scale;
  float* Hdiag;
  uint8_t* Cs;
  float* Wj;
  int8_t* S2;
  int8_t* S3;
  int16_t* Sneed;
  int* Ptile;
  int8_t* Hs;
  int8_t* Hd;
  uint8_t* Qp[2];       // padded copies of Q of the current and of the previous sweep
  uint16_t* Qo;
  float* Apart;
  uint32_t* Flist;      // changed columns per row (fmax each)
  int* Fcnt;
  int* Tstat;
  int* Cbase;           // chunks of changed columns before each row (mpad + 1)
  double* Astate;       // S_i H0 S_i^T per row, the state that later sweeps update
  double* Vstate;       // per row and code: sum of H_jj and sum of G_ij over the code's columns
  int* Nstate;          // per row and code: number of columns
  double* Dpart;        // one C x C slot per chunk of changed columns
  int64_t max_chunks;
  int fmax;
};

// most changed columns per row that a sweep may update instead of summing A_i again
inline int t_fmax(int64_t npad) {
  int64_t f = ceil_div(npad / 2, 32) * 32;      // rows settle at very different speeds: leave room
  if (f < 256) f = 256;
  if (f > 16384) f = 16384;
  return (int)f;
}

inline size_t t_layout(int64_t m, int64_t n, int nbits, char* base, TScratch* out) {
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  const int C = 1 << nbits;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t o_scale = take(4 * sizeof(float));
  const size_t o_diag = take((size_t)n * sizeof(float));
  const size_t o_cs = take((size_t)npad);
  const size_t o_wj = take((size_t)npad * sizeof(float));
  const size_t o_s2 = take((size_t)npad);
  const size_t o_s3 = take((size_t)npad);
  const size_t o_sn = take((size_t)npad * sizeof(int16_t));
  const size_t o_pt = take((size_t)(npad / TM) * sizeof(int));
  const size_t o_hs = take((size_t)TP * npad * npad);
  const size_t o_hd = take((size_t)TP * npad * TM);
  const size_t o_q = take((size_t)mpad * npad);
  const size_t o_q2 = take((size_t)mpad * npad);
  const size_t o_qo = take((size_t)mpad * npad * sizeof(uint16_t));
  const size_t o_ap = take((size_t)t_groups(n) * mpad * C * C * sizeof(float));
  const int fmax = t_fmax(npad);
  const size_t o_fl = take((size_t)mpad * fmax * sizeof(uint32_t));
  const size_t o_fc = take((size_t)mpad * sizeof(int));
  const size_t o_ts = take((8 + 3 * kTLogMax) * sizeof(int));   // counters, then (choice, max, total) per sweep
  const size_t o_as = take((size_t)mpad * C * C * sizeof(double));
  const size_t o_vs = take((size_t)mpad * 2 * C * sizeof(double));
  const size_t o_ns = take((size_t)mpad * C * sizeof(int));
  const size_t o_cb = take((size_t)(mpad + 1) * sizeof(int));
  // a sweep is updated only when at most m n / kDeltaInv indices changed
  const int64_t max_chunks = (m * n / kDeltaInv) / kDeltaChunk + m + 1;
  const size_t o_dp = take((size_t)max_chunks * C * C * sizeof(double));
  if (out != nullptr) {
    out->scale = (float*)(base + o_scale);
    out->Hdiag = (float*)(base + o_diag);
    out->Cs = (uint8_t*)(base + o_cs);
    out->Wj = (float*)(base + o_wj);
    out->S2 = (int8_t*)(base + o_s2);
    out->S3 = (int8_t*)(base + o_s3);
    out->Sneed = (int16_t*)(base + o_sn);
    out->Ptile = (int*)(base + o_pt);
    out->Hs = (int8_t*)(base + o_hs);
    out->Hd = (int8_t*)(base + o_hd);
    out->Qp[0] = (uint8_t*)(base + o_q);
    out->Qp[1] = (uint8_t*)(base + o_q2);
    out->Qo = (uint16_t*)(base + o_qo);
    out->Apart = (float*)(base + o_ap);
    out->Flist = (uint32_t*)(base + o_fl);
    out->Fcnt = (int*)(base + o_fc);
    out->Tstat = (int*)(base + o_ts);
    out->Astate = (double*)(base + o_as);
    out->Vstate = (double*)(base + o_vs);
    out->Nstate = (int*)(base + o_ns);
    out->Cbase = (int*)(base + o_cb);
    out->Dpart = (double*)(base + o_dp);
    out->max_chunks = max_chunks;
    out->fmax = fmax;
  }
  return off;
}

}  // namespace

size_t update_t_scratch_bytes(int64_t m, int64_t n, int nbits) {
  return t_layout(m, n, nbits, nullptr, nullptr);
}

// integer digits of H and their scale factors into scratch (once per layer); allow_delta says
// whether later sweeps of this layer may update A_i from the changed columns
hipError_t launch_t_prepare(hipStream_t s, const float* H, int64_t m, int64_t n, int64_t ldh,
                            int nbits, void* scratch, int allow_delta) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n);
  hipLaunchKernelGGL(t_diag_kernel, dim3(1), dim3(256), 0, s, H, n, ldh, npad, (int)(npad / TM), sc.scale,
                     sc.Hdiag, sc.Cs, sc.Ptile);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(t_rowscale_kernel, dim3((unsigned)n), dim3(256), 0, s, H, n, ldh, sc.scale, sc.Hdiag,
                     sc.Cs, sc.S2, sc.S3, sc.Sneed, sc.Ptile);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the index j of a changed column is stored in 16 bits
  hipLaunchKernelGGL(t_symscale_kernel, dim3(1), dim3(1024), 0, s, sc.Ptile, (int)(npad / TM), n,
                     (allow_delta != 0 && npad <= 65536) ? 1 : 0, sc.Cs, sc.S2, sc.Sneed, sc.Tstat);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(t_split_kernel, dim3((unsigned)ceil_div(npad, 256), (unsigned)npad), dim3(256), 0, s,
                     H, n, ldh, npad, sc.Cs, sc.S2, sc.S3, sc.Ptile, sc.Hs, sc.Hd, sc.Wj);
  return hipGetLastError();
}

// zero-padded aligned copy of Q into buffer `cur` (0 or 1) of scratch
hipError_t launch_t_pad(hipStream_t s, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                        int nbits, void* scratch, int cur) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  const int vec = ((((uintptr_t)Q) & 15) == 0 && (ldq % 16) == 0) ? 1 : 0;
  hipLaunchKernelGGL(pad_q_kernel, dim3((unsigned)ceil_div(npad, 256 * 16), (unsigned)mpad), dim3(256), 0,
                     s, Q, m, n, ldq, npad, nbits, vec, sc.Qp[cur & 1], sc.Qo);
  return hipGetLastError();
}

// columns that changed between the padded copy of the previous sweep (buffer 1 - cur) and the
// current one (buffer cur), per row, with their maximum and total
hipError_t launch_t_flips(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, nbits);
  hipLaunchKernelGGL(t_flips_kernel, dim3((unsigned)mpad), dim3(256), 0, s, sc.Qp[cur & 1], sc.Qp[(cur & 1) ^ 1],
                     npad, sc.fmax, sc.Flist, sc.Fcnt);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(t_chunks_kernel, dim3(1), dim3(1024), 0, s, sc.Fcnt, m, sc.fmax, sc.Cbase, sc.Tstat);
  return hipGetLastError();
}

// partial M_i = sum_{j>k} [Q_ij = a][Q_ik = b] H_jk per group of row tiles (the one-hot GEMM)
template <int NBITS>
static hipError_t launch_t_accum_n(hipStream_t s, int64_t m, int64_t n, void* scratch, int cur) {
  TScratch sc;
  t_layout(m, n, NBITS, (char*)scratch, &sc);
  const int64_t npad = t_npad(n), mpad = t_mpad(m, NBITS);
  const int mtiles = (int)(npad / TM);
  const int groups = t_groups(n);
  const int shmem = T_LDS_BYTES;
  static std::atomic<uint64_t> lds_set{0};
  {
    const hipError_t ea = ensure_dynamic_lds((const void*)t_accum_kernel<NBITS>, shmem, lds_set);
    if (ea != hipSuccess) return ea;
  }
  const int64_t total = (mpad / (TN >> NBITS)) * groups;
  hipLaunchKernelGGL(t_accum_kernel<NBITS>, dim3((unsigned)(8 * ceil_div(total, 8))), dim3(64 * TNW),
                     shmem, s, sc.Hs, sc.Hd, sc.Tstat, sc.fmax, m, n, npad, sc.Qp[cur & 1], sc.Qo, sc.Cs, sc.Wj,
                     sc.Ptile, mpad, mtiles, groups, sc.Apart);
  return hipGetLastError();
}

hipError_t launch_t_accum(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur) {
  switch (nbits) {
    case 1: return launch_t_accum_n<1>(s, m, n, scratch, cur);
    case 2: return launch_t_accum_n<2>(s, m, n, scratch, cur);
    case 3: return launch_t_accum_n<3>(s, m, n, scratch, cur);
    default: return launch_t_accum_n<4>(s, m, n, scratch, cur);
  }
}

// A_i state += the effect of the changed columns (does nothing in a sweep that sums A_i again)
template <int NBITS>
static hipError_t launch_t_delta_n(hipStream_t s, int64_t m, int64_t n, void* scratch, int cur) {
  TScratch sc;
  t_layout(m, n, NBITS, (char*)scratch, &sc);
  const int64_t npad = t_npad(n);
  hipLaunchKernelGGL(t_delta_kernel<NBITS>, dim3((unsigned)ceil_div(sc.max_chunks, 4)), dim3(256), 0, s, sc.Hs,
                     npad, sc.Qp[cur & 1], sc.Qp[(cur & 1) ^ 1], sc.Cs, sc.Wj, sc.Flist, sc.Fcnt, sc.Cbase, sc.Tstat,
                     sc.fmax, m, n, sc.Dpart);
  return hipGetLastError();
}

hipError_t launch_t_delta(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur) {
  switch (nbits) {
    case 1: return launch_t_delta_n<1>(s, m, n, scratch, cur);
    case 2: return launch_t_delta_n<2>(s, m, n, scratch, cur);
    case 3: return launch_t_delta_n<3>(s, m, n, scratch, cur);
    default: return launch_t_delta_n<4>(s, m, n, scratch, cur);
  }
}

// assemble A_i, b_i and solve; G = W H
hipError_t launch_t_solve(hipStream_t s, const float* G, int64_t ldg, int64_t m, int64_t n,
                          const uint8_t* Q, int64_t ldq, int nbits, int empty_mode, float* T,
                          int32_t* empty_count, void* scratch, int sweep) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  const int64_t mpad = t_mpad(m, nbits);
  int* tlog = (sweep >= 0 && sweep < kTLogMax) ? sc.Tstat + 8 + 3 * sweep : nullptr;
  hipLaunchKernelGGL(t_solve_kernel, dim3((unsigned)m), dim3(64), 0, s, sc.Apart, t_groups(n), sc.Tstat, sc.fmax,
                     m, sc.Astate, tlog, sc.Cbase, sc.Dpart, sc.Vstate, sc.Nstate, sc.Flist, sc.Fcnt, mpad, sc.scale,
                     sc.Hdiag, G, ldg, Q, ldq, n, nbits,
                     empty_mode, T, empty_count);
  return hipGetLastError();
}

hipError_t read_t_log(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int* modes_host, int count) {
  TScratch sc;
  t_layout(m, n, nbits, (char*)scratch, &sc);
  if (count > kTLogMax) count = kTLogMax;
  hipError_t e = hipMemcpyAsync(modes_host, sc.Tstat + 8, (size_t)count * 3 * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(s);
}

}  // namespace ganq
