// Deployment side of GANQ: the stored form of a quantized layer (N-bit codes plus
// a 2^N-entry fp16 table per row, Table 1) and the look-up-table product for one
// activation vector, y_i = sum_j T_i[Q_ij] x_j (Figure 1(a), right; batch-1
// decoding of Section 4.4), optionally plus the sparse outlier part of GANQ*
// (Section 3.3).
//
// Stored codes: row i is a little-endian bit stream, code j in bits [N j, N j + N).
// 32 codes are 4 N bytes, which is what one lane fetches at a time, so a wavefront
// covers 2048 columns ("segment") per fetch and a row needs no padding beyond the
// last group of 32.
//
// The codes stream from HBM once; what has to keep up with them is the table
// look-up.  The 16 rows' tables sit in LDS.  At N = 4 a table has one entry per bank
// (fp16 in the low half of a 4-byte word, rows 64 bytes apart): a look-up
// instruction of a wavefront reads one row's table, so its at most 16 distinct
// addresses fall into 16 distinct banks and it never conflicts; the entry meets its
// activation in a mixed fp16 x fp16 -> fp32 fused multiply-add, exact in the
// product.  At N <= 3 two adjacent codes are looked up at once in a table of all
// 4^N ordered pairs (at most 64 words, two per bank) and meet their two activations
// in one v_dot2_f32_f16: half the LDS reads and half the arithmetic per code (at
// N = 4 the 256 words of such a table collide in the banks: measured slower).  The
// byte offset of an entry is cut out of the code words with masked copies of a whole
// word and one byte extraction per look-up where fields do not straddle bytes.  Look-ups
// run one batch ahead of the multiply-adds.  A workgroup owns 16 whole rows; its 8
// wavefronts are arranged as (row group) x (segment lane), the segment lanes
// striding over the segments of a row.  Per-lane partial sums are reduced once per
// row at the end, the segment lanes' sums are added in a fixed order through LDS:
// results are bit-reproducible.  On the large layers the kernel is bound by LDS
// instruction issue and vector ALU work per code, not by HBM.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int GR = 16;       // rows per workgroup
constexpr int GNW = 8;       // wavefronts per workgroup
constexpr int GSEG = 2048;   // columns per wavefront fetch: 64 lanes x 32 codes

typedef _Float16 half2v __attribute__((ext_vector_type(2)));

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One 32-code group (N words) from global memory, as one vector load.
template <int N>
__device__ inline void load_group(const uint32_t* __restrict__ p, uint32_t (&d)[N]) {
  if constexpr (N == 4) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
  } else if constexpr (N == 3) {
    struct __attribute__((packed, aligned(4))) U3 { uint32_t a, b, c; };
    const U3 v = *reinterpret_cast<const U3*>(p);
    d[0] = v.a; d[1] = v.b; d[2] = v.c;
  } else if constexpr (N == 2) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    d[0] = v.x; d[1] = v.y;
  } else {
    d[0] = *p;
  }
}

// Byte offsets (4 * field value) of the F-bit fields of a 32-code group held in NW words: a
// field is one code (F = N) or two adjacent codes (F = 2 N).
// F = 1, 2, 4: a field never straddles a byte, so the word is masked once per position of a
// field within a byte (all four bytes at a time, 2 operations per 4 fields) and each field then
// costs one byte extraction; the empty asm keeps the compiler from folding the two steps back
// into a shift and a mask per field.  F = 6: shift and mask per field, a funnel shift where a
// field straddles two words.
template <int F, int NW>
struct FieldOffsets {
  static constexpr bool BYTEWISE = (8 % F) == 0;
  static constexpr int PB = BYTEWISE ? 8 / F : 1;      // field positions within a byte
  static constexpr uint32_t MASK = ((1u << F) - 1u) << 2;
  uint32_t mk[NW][PB];
  uint32_t raw[NW];
  __device__ inline explicit FieldOffsets(const uint32_t (&d)[NW]) {
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      raw[w] = d[w];
      if constexpr (BYTEWISE) {
#pragma unroll
        for (int ps = 0; ps < PB; ++ps) {
          uint32_t v = ((F * ps < 2) ? (d[w] << (2 - F * ps)) : (d[w] >> (F * ps - 2))) & (MASK * 0x01010101u);
          asm("" : "+v"(v));
          mk[w][ps] = v;
        }
      }
    }
  }
  __device__ inline uint32_t at(int j) const {
    const int bit = F * j;
    const int w = bit >> 5, sh = bit & 31;
    if constexpr (BYTEWISE) {
      return (mk[w][(sh & 7) / F] >> (8 * (sh >> 3))) & 0xffu;
    } else {
      if (sh + F > 32) {
        const uint32_t v = __builtin_amdgcn_alignbit(raw[(w + 1 < NW) ? w + 1 : w], raw[w], sh);
        return (v << 2) & MASK;
      }
      if (sh < 2) return (raw[w] << (2 - sh)) & MASK;
      return (raw[w] >> (sh - 2)) & MASK;
    }
  }
};

// SW = segment lanes (1, 2, 4 or 8 wavefronts side by side on one row); the other
// 8 / SW wavefronts take different rows, so every wavefront owns 2 SW of the 16 rows.
template <int N, int SW>
__global__ __launch_bounds__(64 * GNW, 4) void lut_gemv_kernel(
    const uint8_t* __restrict__ packed, int64_t ldp, const uint16_t* __restrict__ lut, int64_t m,
    int64_t n, const _Float16* __restrict__ x, float* __restrict__ y,
    const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const float* __restrict__ values) {
  constexpr int C = 1 << N;
  constexpr int RG = GNW / SW;      // row groups
  constexpr int RPW = GR / RG;      // rows per wavefront
  // N <= 3: codes are looked up in pairs, in a table of all 4^N ordered pairs (T[a], T[b]) as
  // packed fp16 pairs (at most 64 words per row: two per bank); N = 4: one by one (256 words
  // would collide in the banks), the entry in the low half of a word.
  constexpr bool PAIR = N <= 3;
  constexpr int F = PAIR ? 2 * N : N;          // bits per look-up
  constexpr int TW = 1 << F;                   // table words per row
  constexpr int LPG = 32 * N / F;              // look-ups per 32-code group
  __shared__ __attribute__((aligned(16))) uint32_t tab[GR][TW];
  __shared__ float part[SW][GR];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sl = wave % SW, g = (RG == 1) ? 0 : wave / SW;
  const int64_t row0 = (int64_t)blockIdx.x * GR;

  // the 16 rows' tables
  for (int e = tid; e < GR * TW; e += 64 * GNW) {
    const int r = e / TW, idx = e % TW;
    uint32_t v = 0u;
    if (row0 + r < m) {
      const uint16_t* lr = lut + (row0 + r) * C;
      v = PAIR ? ((uint32_t)lr[idx & (C - 1)] | ((uint32_t)lr[idx >> N] << 16)) : (uint32_t)lr[idx];
    }
    tab[r][idx] = v;
  }
  const uint32_t gbase = (uint32_t)g * (TW * 4u);   // this wavefront's rows are g, g + RG, ...
  __syncthreads();

  float acc[RPW];
#pragma unroll
  for (int k = 0; k < RPW; ++k) acc[k] = 0.f;

  const int64_t nseg = ceil_div(n, GSEG);
  for (int64_t seg = sl; seg < nseg; seg += SW) {
    const int64_t col0 = seg * GSEG + (int64_t)lane * 32;
    // this lane's 32 activations as 16 fp16 pairs; columns >= n count as zero
    uint32_t xr[16];
    if (col0 + 32 <= n && ((uintptr_t)x & 15) == 0) {
      const uint4* xp = reinterpret_cast<const uint4*>(x + col0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint4 t = xp[u];
        xr[4 * u] = t.x; xr[4 * u + 1] = t.y; xr[4 * u + 2] = t.z; xr[4 * u + 3] = t.w;
      }
    } else {
      const uint16_t* xs = reinterpret_cast<const uint16_t*>(x);
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int64_t c = col0 + 2 * u;
        const uint32_t lo = (c < n) ? xs[c] : 0u, hi = (c + 1 < n) ? xs[c + 1] : 0u;
        xr[u] = lo | (hi << 16);
      }
    }
    // the code groups of this wavefront's rows, all fetched before any is used; a lane whose
    // group lies outside the matrix fetches group 0 of row 0 instead and discards it
    uint32_t q[RPW][N];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const int64_t row = row0 + g + RG * k;
      const bool ok = row < m && col0 < n;
      const uint32_t* src = reinterpret_cast<const uint32_t*>(packed + (ok ? row : 0) * ldp) +
                            (ok ? (seg * 64 + lane) * N : 0);
      load_group<N>(src, q[k]);
#pragma unroll
      for (int w = 0; w < N; ++w) q[k][w] = ok ? q[k][w] : 0u;
    }
    // Look-ups in batches (LB per row, two rows): the reads of the next batch are issued
    // before the previous batch is multiplied, and the scheduling barriers keep it that way
    // (left alone, the compiler waits for every single read).  The two rows' multiply-adds
    // alternate, so consecutive instructions do not depend on each other.
    constexpr int LB = (RPW * N >= 64) ? 4 : 8;     // look-ups per row and batch (register budget)
    constexpr int BPR = LPG / LB;                   // batches per pair of rows
    constexpr int NB = (RPW / 2) * BPR;
    uint32_t ev[2][2 * LB];
    auto lookup = [&](int bt, uint32_t (&e)[2 * LB]) {
      const int kp = bt / BPR, h = bt % BPR;
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int k = 2 * kp + rr;
        const char* t = reinterpret_cast<const char*>(tab[RG * k]);
        const FieldOffsets<F, N> off(q[k]);
#pragma unroll
        for (int j = 0; j < LB; ++j) {
          const uint32_t o = off.at(LB * h + j) | gbase;
          if constexpr (PAIR)
            e[LB * rr + j] = *reinterpret_cast<const uint32_t*>(t + o);
          else
            e[LB * rr + j] = *reinterpret_cast<const uint16_t*>(t + o);
        }
      }
    };
    lookup(0, ev[0]);
#pragma unroll
    for (int bt = 0; bt < NB; ++bt) {
      __builtin_amdgcn_sched_barrier(0);
      if (bt + 1 < NB) lookup(bt + 1, ev[(bt + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
      const int kp = bt / BPR, h = bt % BPR;
      float a0 = acc[2 * kp], a1 = acc[2 * kp + 1];
#pragma unroll
      for (int j = 0; j < LB; ++j) {
        const int l = LB * h + j;                   // look-up within the group
        if constexpr (PAIR) {
          const half2v xx = __builtin_bit_cast(half2v, xr[l]);
          a0 = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, ev[bt & 1][j]), xx, a0, false);
          a1 = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, ev[bt & 1][LB + j]), xx, a1, false);
        } else {
          const half2v xx = __builtin_bit_cast(half2v, xr[l >> 1]);
          const half2v e0 = __builtin_bit_cast(half2v, ev[bt & 1][j]);
          const half2v e1 = __builtin_bit_cast(half2v, ev[bt & 1][LB + j]);
          a0 = fmaf((float)e0[0], (float)xx[l & 1], a0);
          a1 = fmaf((float)e1[0], (float)xx[l & 1], a1);
        }
      }
      acc[2 * kp] = a0;
      acc[2 * kp + 1] = a1;
    }
  }

  // sparse part: the first segment lane of each row group adds its rows' outliers
  if (row_ptr != nullptr && sl == 0) {
    const uint16_t* xs = reinterpret_cast<const uint16_t*>(x);
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const int64_t row = row0 + g + RG * k;
      if (row < m) {
        const int64_t e1 = row_ptr[row + 1];
        float a = acc[k];
        for (int64_t e = row_ptr[row] + lane; e < e1; e += 64) {
          const _Float16 xv = __builtin_bit_cast(_Float16, xs[col_idx[e]]);
          a = fmaf(values[e], (float)xv, a);
        }
        acc[k] = a;
      }
    }
  }

#pragma unroll
  for (int k = 0; k < RPW; ++k) {
    const float v = wave_sum(acc[k]);
    if (lane == 0) part[sl][g + RG * k] = v;
  }
  __syncthreads();
  if (tid < GR && row0 + tid < m) {
    float v = part[0][tid];
#pragma unroll
    for (int s2 = 1; s2 < SW; ++s2) v += part[s2][tid];
    y[row0 + tid] = v;
  }
}

// One thread packs 32 codes into N words; thread (0, row) also rounds the row's table to fp16.
template <int N>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ Q, int64_t n, int64_t ldq,
                                                   const float* __restrict__ T,
                                                   uint8_t* __restrict__ packed, int64_t ldp,
                                                   int64_t row_bytes, uint16_t* __restrict__ lut) {
  constexpr int C = 1 << N;
  const int64_t row = blockIdx.y;
  const int64_t grp = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t ngrp = ceil_div(n, 32);
  if (blockIdx.x == 0 && threadIdx.x < C) {
    const _Float16 h = (_Float16)T[row * C + threadIdx.x];     // round to nearest even
    lut[row * C + threadIdx.x] = __builtin_bit_cast(uint16_t, h);
  }
  if (grp >= ngrp) return;
  const uint8_t* src = Q + row * ldq + grp * 32;
  uint32_t out[N];
#pragma unroll
  for (int w = 0; w < N; ++w) out[w] = 0u;
  uint32_t in[8];       // the 32 codes, four per word
  if (grp * 32 + 32 <= n && ((uintptr_t)src & 15) == 0) {
    const uint4 a = reinterpret_cast<const uint4*>(src)[0], b = reinterpret_cast<const uint4*>(src)[1];
    in[0] = a.x; in[1] = a.y; in[2] = a.z; in[3] = a.w;
    in[4] = b.x; in[5] = b.y; in[6] = b.z; in[7] = b.w;
  } else {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      in[u] = 0u;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if (grp * 32 + 4 * u + b < n) in[u] |= (uint32_t)src[4 * u + b] << (8 * b);
    }
  }
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const uint32_t c = (in[j >> 2] >> (8 * (j & 3))) & (C - 1);
    const int bit = N * j, w = bit >> 5, sh = bit & 31;
    out[w] |= c << sh;
    if (sh + N > 32) out[w + 1 < N ? w + 1 : w] |= c >> (32 - sh);
  }
  uint32_t* dst = reinterpret_cast<uint32_t*>(packed + row * ldp) + grp * N;
#pragma unroll
  for (int w = 0; w < N; ++w) dst[w] = out[w];
  if (grp == ngrp - 1) {       // zero the alignment padding of the row
    for (int64_t b = ngrp * 4 * N; b < row_bytes; b += 4)
      *reinterpret_cast<uint32_t*>(packed + row * ldp + b) = 0u;
  }
}

template <int N>
hipError_t launch_gemv_n(hipStream_t s, const uint8_t* packed, int64_t ldp, const uint16_t* lut, int64_t m,
                         int64_t n, const _Float16* x, float* y, const int64_t* row_ptr,
                         const int32_t* col_idx, const float* values) {
  const int64_t nseg = ceil_div(n, GSEG);
  const dim3 grid((unsigned)ceil_div(m, GR)), block(64 * GNW);
  // segment lanes: the widest arrangement among those that leave the fewest lanes idle in the
  // last round over the segments
  int sw = 1;
  int64_t best = nseg;                       // slots used with one lane: no idle slot
  for (int c = 2; c <= 8; c *= 2) {
    const int64_t slots = ceil_div(nseg, c) * c;
    if (slots <= best) { best = slots; sw = c; }
  }
  if (sw == 8)
    hipLaunchKernelGGL((lut_gemv_kernel<N, 8>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  else if (sw == 4)
    hipLaunchKernelGGL((lut_gemv_kernel<N, 4>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  else if (sw == 2)
    hipLaunchKernelGGL((lut_gemv_kernel<N, 2>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  else
    hipLaunchKernelGGL((lut_gemv_kernel<N, 1>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  return hipGetLastError();
}

}  // namespace

int64_t packed_row_bytes(int64_t n, int nbits) {
  return (ceil_div(n, 32) * 4 * nbits + 15) / 16 * 16;
}

// Requires 1 <= nbits <= 4, ldp % 4 == 0, ldp >= packed_row_bytes(n, nbits), m <= 65535 (grid.y).
hipError_t launch_pack_layer(hipStream_t s, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                             const float* T, int nbits, uint8_t* packed, int64_t ldp, uint16_t* lut) {
  const dim3 grid((unsigned)ceil_div(ceil_div(n, 32), 256), (unsigned)m), block(256);
  const int64_t rb = packed_row_bytes(n, nbits);
  switch (nbits) {
    case 1: hipLaunchKernelGGL(pack_kernel<1>, grid, block, 0, s, Q, n, ldq, T, packed, ldp, rb, lut); break;
    case 2: hipLaunchKernelGGL(pack_kernel<2>, grid, block, 0, s, Q, n, ldq, T, packed, ldp, rb, lut); break;
    case 3: hipLaunchKernelGGL(pack_kernel<3>, grid, block, 0, s, Q, n, ldq, T, packed, ldp, rb, lut); break;
    default: hipLaunchKernelGGL(pack_kernel<4>, grid, block, 0, s, Q, n, ldq, T, packed, ldp, rb, lut); break;
  }
  return hipGetLastError();
}

// Requires 1 <= nbits <= 4, ldp % 4 == 0, packed 4-byte aligned, ldp >= packed_row_bytes(n, nbits).
hipError_t launch_lut_gemv(hipStream_t s, const uint8_t* packed, int64_t ldp, const uint16_t* lut, int nbits,
                           int64_t m, int64_t n, const _Float16* x, float* y, const int64_t* row_ptr,
                           const int32_t* col_idx, const float* values) {
  switch (nbits) {
    case 1: return launch_gemv_n<1>(s, packed, ldp, lut, m, n, x, y, row_ptr, col_idx, values);
    case 2: return launch_gemv_n<2>(s, packed, ldp, lut, m, n, x, y, row_ptr, col_idx, values);
    case 3: return launch_gemv_n<3>(s, packed, ldp, lut, m, n, x, y, row_ptr, col_idx, values);
    default: return launch_gemv_n<4>(s, packed, ldp, lut, m, n, x, y, row_ptr, col_idx, values);
  }
}

}  // namespace ganq
