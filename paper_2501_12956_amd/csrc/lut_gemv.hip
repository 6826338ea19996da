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
// The product is bound by the stream of codes from HBM; what has to keep up with
// it is the table look-up.  Looking codes up in pairs halves the LDS operations:
// the workgroup first expands each of its 16 rows' tables into a table of all 4^N
// ordered pairs (T[a], T[b]) as packed fp16 pairs, indexed by the 2N bits of two
// adjacent codes, so one 4-byte LDS read feeds one v_dot2_f32_f16 against the
// matching pair of activations (fp32 accumulation).  A workgroup owns 16 whole
// rows; its 8 wavefronts are arranged as (row group) x (segment lane), the segment
// lanes striding over the segments of a row.  Per-lane partial sums are reduced
// once per row at the end, the segment lanes' sums are added in a fixed order
// through LDS: results are bit-reproducible.
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

// The 2N bits of code pair p (codes 2p and 2p + 1) of a 32-code group held in d[0..N).
template <int N>
__device__ inline uint32_t pair_index(const uint32_t (&d)[N], int p) {
  const int bit = 2 * N * p;
  const int w = bit >> 5, sh = bit & 31;
  uint32_t v = d[w] >> sh;
  if (sh + 2 * N > 32) v |= d[(w + 1 < N) ? w + 1 : w] << (32 - sh);   // straddles two words (N = 3)
  return v & ((1u << (2 * N)) - 1u);
}

// SW = segment lanes (1, 2, 4 or 8 wavefronts side by side on one row); the other
// 8 / SW wavefronts take different rows, so every wavefront owns 2 SW of the 16 rows.
template <int N, int SW>
__global__ __launch_bounds__(64 * GNW) void lut_gemv_kernel(
    const uint8_t* __restrict__ packed, int64_t ldp, const uint16_t* __restrict__ lut, int64_t m,
    int64_t n, const _Float16* __restrict__ x, float* __restrict__ y,
    const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const float* __restrict__ values) {
  constexpr int C = 1 << N, PT = C * C;
  constexpr int RG = GNW / SW;      // row groups
  constexpr int RPW = GR / RG;      // rows per wavefront
  __shared__ uint32_t tab[GR][PT];
  __shared__ float part[SW][GR];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sl = wave % SW, g = wave / SW;
  const int64_t row0 = (int64_t)blockIdx.x * GR;

  // pair tables of the 16 rows: entry (b << N | a) = (T[a], T[b]) as two fp16
  for (int e = tid; e < GR * PT; e += 64 * GNW) {
    const int r = e / PT, idx = e % PT;
    const int64_t row = row0 + r;
    uint32_t v = 0;
    if (row < m) v = (uint32_t)lut[row * C + (idx & (C - 1))] | ((uint32_t)lut[row * C + (idx >> N)] << 16);
    tab[r][idx] = v;
  }
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
    // the code groups of this wavefront's rows, all fetched before any is used
    uint32_t q[RPW][N];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const int64_t row = row0 + g + RG * k;
      const bool ok = row < m && col0 < n;
      const uint32_t* src =
          reinterpret_cast<const uint32_t*>(packed + row * ldp) + (seg * 64 + lane) * N;
#pragma unroll
      for (int w = 0; w < N; ++w) q[k][w] = ok ? src[w] : 0u;
    }
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const uint32_t* t = tab[g + RG * k];
      float a = acc[k];
#pragma unroll
      for (int p = 0; p < 16; ++p) {
        const uint32_t e = t[pair_index<N>(q[k], p)];
        a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, e), __builtin_bit_cast(half2v, xr[p]), a,
                                   false);
      }
      acc[k] = a;
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
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const uint32_t c = (grp * 32 + j < n) ? (uint32_t)(src[j] & (C - 1)) : 0u;
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
  if (nseg >= 8)
    hipLaunchKernelGGL((lut_gemv_kernel<N, 8>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  else if (nseg >= 4)
    hipLaunchKernelGGL((lut_gemv_kernel<N, 4>), grid, block, 0, s, packed, ldp, lut, m, n, x, y, row_ptr,
                       col_idx, values);
  else if (nseg >= 2)
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
