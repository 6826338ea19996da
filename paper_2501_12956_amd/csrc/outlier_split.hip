// Outlier split W = W_sparse + W_dense (Appendix B, Algorithm 2; Section 3.3):
// per row, the entries at or beyond the two symmetric tail cut-offs - the values
// at sorted positions `lower` and `upper` of the row, comparisons <= and >= -
// go to W_sparse (returned as CSR, columns ascending), the rest to W_dense,
// which keeps zeros at the outlier positions.  No arithmetic on the values:
// the split is exact.
//
// Three kernels: (1) one workgroup per row sorts the row in LDS (bitonic
// network) and records the two cut-off values and the number of outliers;
// (2) one workgroup turns the counts into row offsets; (3) one workgroup per
// row writes W_dense and compacts the outliers in column order (ballot-based
// scan).  Bound by HBM: the row is read twice, W_dense written once.
#include "ganq_internal.h"

namespace ganq {
namespace {

template <typename TW>
__global__ __launch_bounds__(1024) void outlier_cut_kernel(const TW* __restrict__ W, int64_t n,
                                                           int64_t ldw, int npow2, int lower, int upper,
                                                           float* __restrict__ cuts,
                                                           int32_t* __restrict__ counts) {
  extern __shared__ float srt[];
  __shared__ int wsum[16];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  for (int e = tid; e < npow2; e += 1024)
    srt[e] = (e < n) ? (float)W[row * ldw + e] : __builtin_huge_valf();
  __syncthreads();
  bitonic_sort_lds_1024(srt, npow2, tid);
  const float c_lo = srt[lower], c_up = srt[upper];
  int cnt = 0;
  for (int e = tid; e < n; e += 1024) {
    const float w = (float)W[row * ldw + e];
    cnt += (w >= c_up || w <= c_lo) ? 1 : 0;
  }
  for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off);
  if ((tid & 63) == 0) wsum[tid >> 6] = cnt;
  __syncthreads();
  if (tid == 0) {
    int total = 0;
    for (int w = 0; w < 16; ++w) total += wsum[w];
    counts[row] = total;
    cuts[2 * row] = c_lo;
    cuts[2 * row + 1] = c_up;
  }
}

// row_ptr[0] = 0, row_ptr[i + 1] = counts[0] + .. + counts[i]
__global__ __launch_bounds__(1024) void outlier_scan_kernel(const int32_t* __restrict__ counts, int64_t m,
                                                            int64_t* __restrict__ row_ptr) {
  __shared__ int64_t part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (m + 1023) / 1024;
  const int64_t b = tid * per, e = (b + per < m) ? b + per : m;
  int64_t s = 0;
  for (int64_t i = b; i < e; ++i) s += counts[i];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) {
    int64_t run = 0;
    for (int t = 0; t < 1024; ++t) {
      const int64_t v = part[t];
      part[t] = run;
      run += v;
    }
    row_ptr[0] = 0;
  }
  __syncthreads();
  int64_t run = part[tid];
  for (int64_t i = b; i < e; ++i) {
    run += counts[i];
    row_ptr[i + 1] = run;
  }
}

template <typename TW>
__global__ __launch_bounds__(256) void outlier_emit_kernel(const TW* __restrict__ W, int64_t n, int64_t ldw,
                                                           const float* __restrict__ cuts,
                                                           const int64_t* __restrict__ row_ptr,
                                                           float* __restrict__ Wd, int64_t ldd,
                                                           int32_t* __restrict__ col_idx,
                                                           float* __restrict__ values, int64_t capacity) {
  __shared__ int wcnt[4];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float c_lo = cuts[2 * row], c_up = cuts[2 * row + 1];
  int64_t base = row_ptr[row];
  for (int64_t c0 = 0; c0 < n; c0 += 256) {
    const int64_t c = c0 + tid;
    const float w = (c < n) ? (float)W[row * ldw + c] : 0.f;
    const bool out = c < n && (w >= c_up || w <= c_lo);
    if (c < n) Wd[row * ldd + c] = out ? 0.f : w;
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(out);
    const int before = __builtin_popcountll(vote & ((1ull << lane) - 1ull));
    if (lane == 0) wcnt[wave] = __builtin_popcountll(vote);
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      woff += (v < wave) ? wcnt[v] : 0;
      total += wcnt[v];
    }
    if (out) {
      const int64_t pos = base + woff + before;
      if (pos < capacity) {
        col_idx[pos] = (int32_t)c;
        values[pos] = w;
      }
    }
    base += total;
    __syncthreads();
  }
}

}  // namespace

size_t outlier_scratch_bytes(int64_t m) {
  return align_up((size_t)m * 2 * sizeof(float)) + align_up((size_t)m * sizeof(int32_t));
}

// scratch: [cuts m x 2 float][counts m int32]
hipError_t launch_outlier_split(hipStream_t s, const void* W, int w_is_f16, int64_t m, int64_t n, int64_t ldw,
                                int lower, int upper, float* Wd, int64_t ldd, int64_t* row_ptr,
                                int32_t* col_idx, float* values, int64_t capacity, void* scratch) {
  float* cuts = (float*)scratch;
  int32_t* counts = (int32_t*)((char*)scratch + align_up((size_t)m * 2 * sizeof(float)));
  int npow2 = 1;
  while (npow2 < n) npow2 <<= 1;
  const size_t shmem = (size_t)npow2 * sizeof(float);
  hipError_t e;
  if (w_is_f16) {
    auto kern = outlier_cut_kernel<_Float16>;
    if (shmem > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)m), dim3(1024), shmem, s, (const _Float16*)W, n, ldw, npow2, lower,
                       upper, cuts, counts);
  } else {
    auto kern = outlier_cut_kernel<float>;
    if (shmem > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)m), dim3(1024), shmem, s, (const float*)W, n, ldw, npow2, lower,
                       upper, cuts, counts);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(outlier_scan_kernel, dim3(1), dim3(1024), 0, s, counts, m, row_ptr);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (w_is_f16)
    hipLaunchKernelGGL(outlier_emit_kernel<_Float16>, dim3((unsigned)m), dim3(256), 0, s, (const _Float16*)W, n,
                       ldw, cuts, row_ptr, Wd, ldd, col_idx, values, capacity);
  else
    hipLaunchKernelGGL(outlier_emit_kernel<float>, dim3((unsigned)m), dim3(256), 0, s, (const float*)W, n, ldw,
                       cuts, row_ptr, Wd, ldd, col_idx, values, capacity);
  return hipGetLastError();
}

}  // namespace ganq
