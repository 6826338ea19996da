// Internal declarations shared by the host-side C ABI and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include <atomic>

#include "ganq.h"

struct ganq_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  bool device_ready = false;
  std::string last_error;
  // optional per-kernel-class timing with HIP events on the context's stream
  bool prof_on = false;
  struct ProfRec { int cls; hipEvent_t a, b; int tag; };
  std::vector<ProfRec> prof_pending;
  std::vector<hipEvent_t> prof_free;
  double prof_ms[GANQ_K_COUNT] = {0};
  int64_t prof_launches[GANQ_K_COUNT] = {0};
  // second stream (default priority) and two events: work of one call that does not depend on
  // the factorisation runs beside it; always joined before the call returns
  // log of the last ganq_quantize_layer call (3 ints per sweep, see read_t_log) and its length
  int sweep_log[3 * 64] = {0};
  int sweep_log_len = 0;
  // Per-layer inputs of the stand-alone T-update kept at the start of the workspace between calls
  // (ganq_update_T_prepare): G = W H, the integer digits of H and their scratch.  While valid, the
  // other stand-alone calls carve their scratch behind these `bytes`.
  struct TPrep {
    bool valid = false;
    const void* W = nullptr;
    const void* H = nullptr;
    int64_t ldw = 0, ldh = 0, m = 0, n = 0;
    int nbits = 0;
    void* ws = nullptr;
    size_t bytes = 0;
    float* G = nullptr;
    void* t_scratch = nullptr;
  } tprep;
  hipStream_t side = nullptr;
  hipEvent_t fork_ev = nullptr, join_ev = nullptr;
};

namespace ganq {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

typedef int int4v __attribute__((ext_vector_type(4)));

// Raw buffer descriptor over [base, base + bytes): a load whose offset falls outside reads zero.
__device__ inline int4v make_rsrc(const void* base, int64_t bytes) {
  const uint64_t ad = (uint64_t)(uintptr_t)base;
  int4v r;
  r[0] = (int)(uint32_t)ad;
  r[1] = (int)(uint32_t)((ad >> 32) & 0xffffu);
  r[2] = (int)(uint32_t)bytes;
  r[3] = 0x00020000;
  return r;
}
// One wavefront-wide load from global memory straight into LDS: lane l's 16 bytes land at LDS
// byte lds_addr + 16 l.  The compiler does not see these loads, so its own vmcnt waits can only
// be too early for them, never for its own loads (the counter retires in order); a kernel waits
// for them explicitly (wait_all_loads) before the barrier that publishes a stage.
__device__ inline void load16_to_lds(int4v rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
__device__ inline void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int64_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + (kAlign - 1)) & ~(size_t)(kAlign - 1); }
__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Ascending bitonic sort of npow2 (a power of two) floats in LDS by a workgroup of 1024
// threads; the caller has filled srt and synchronised.  Wavefront w owns the elements
// [256 w', 256 w' + 256) for w' = w, w + 16, ...: a step whose partner distance j is below 256
// stays inside such a segment, so it needs no workgroup barrier - the LDS operations of one
// wavefront execute in order, and the wave barrier only keeps the compiler from moving them.
// Only the steps with j >= 256 (10 of the 78 for 4096 elements) synchronise the workgroup.
// Returns after a workgroup barrier.
__device__ inline void bitonic_sort_lds_1024(float* srt, int npow2, int tid) {
  const int wv = tid >> 6, ln = tid & 63;
  for (int k = 2; k <= npow2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      // compare-exchange t pairs elements e (bit log2(j) clear) and e | j: every lane is busy, and
      // the 128 exchanges 128 S .. 128 S + 127 stay inside segment S when j < 256
      for (int sg = wv; sg * 256 < npow2; sg += 16) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int t = 128 * sg + 64 * u + ln;
          const int e = ((t & ~(j - 1)) << 1) | (t & (j - 1));
          const int partner = e | j;
          if (partner < npow2) {
            const bool up = (e & k) == 0;
            const float a = srt[e], b = srt[partner];
            if ((a > b) == up) {
              srt[e] = b;
              srt[partner] = a;
            }
          }
        }
      }
      if (j >= 256 || (j >> 1) >= 256 || (j == 1 && k >= 256))
        __syncthreads();          // this step or the next one crosses segments
      else
        __builtin_amdgcn_wave_barrier();
    }
  }
  __syncthreads();
}

// Raises a kernel's dynamic LDS limit once per device (the attribute is per device; `done`
// holds one bit per device ordinal and belongs to that kernel's launcher).
inline hipError_t ensure_dynamic_lds(const void* fn, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Bump allocator over the caller's workspace.
struct Arena {
  char* base;
  size_t cap;
  size_t off = 0;
  Arena(void* p, size_t bytes) : base((char*)p), cap(bytes) {}
  void* take(size_t bytes) {
    size_t a = align_up(off);
    if (base == nullptr || a + bytes > cap) return nullptr;
    off = a + bytes;
    return base + a;
  }
};

// ---- sizes of scratch regions (shared by ganq_workspace_bytes and the calls) ----
constexpr int kSlabRows = 16;       // rows per workgroup in the S-update
constexpr int kHessTile = 256;      // output tile edge of the fp16 H = X X^T kernel
constexpr int kHessMaxSplit = 16;   // upper bound on token-axis splits

inline int64_t pad_rows(int64_t m) { return ceil_div(m, kSlabRows) * kSlabRows; }
int hessian_split(int64_t n, int64_t p);
size_t hessian_scratch_bytes(int64_t n, int64_t p);
constexpr int64_t kTokenChunk = 32768;   // tokens transposed at a time by the token-major entry point
bool hessian_tokens_direct_ok(const void* Xt, int64_t n, int64_t p, int64_t ldxt);
hipError_t launch_hessian_f16_tokens(hipStream_t s, const _Float16* Xt, int64_t n, int64_t p, int64_t ldxt,
                                     float* H, int64_t ldh, int accumulate, float* partials);
hipError_t launch_transpose_tokens(hipStream_t s, const void* Xt, int elem_bytes, int64_t pc, int64_t n,
                                   int64_t ldxt, void* Xn, int64_t ldn);
size_t update_s_scratch_bytes(int64_t m, int64_t n);
size_t update_t_scratch_bytes(int64_t m, int64_t n, int nbits);
size_t loss_scratch_bytes(int64_t m, int64_t n);
size_t cholesky_scratch_bytes(int64_t n);
size_t outlier_scratch_bytes(int64_t m);
size_t gemm_split_scratch_bytes(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemm_split(hipStream_t s, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
                             const float* B, int64_t ldb, float* C, int64_t ldc, void* scratch, int b_ready);
hipError_t launch_outlier_split(hipStream_t s, const void* W, int w_is_f16, int64_t m, int64_t n, int64_t ldw,
                                int lower, int upper, float* Wd, int64_t ldd, int64_t* row_ptr,
                                int32_t* col_idx, float* values, int64_t capacity, void* scratch);
int64_t packed_row_bytes(int64_t n, int nbits);
hipError_t launch_pack_layer(hipStream_t s, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                             const float* T, int nbits, uint8_t* packed, int64_t ldp, uint16_t* lut);
hipError_t launch_lut_gemv(hipStream_t s, const uint8_t* packed, int64_t ldp, const uint16_t* lut, int nbits,
                           int64_t m, int64_t n, const _Float16* x, float* y, const int64_t* row_ptr,
                           const int32_t* col_idx, const float* values);

hipError_t launch_peak_probe(hipStream_t s, int which, void* buf, size_t bytes, double* ops);

// ---- kernel launchers (all enqueue on `s`, return the HIP error of the launch) ----

// C = alpha * A * op(B) + beta * C, fp32 on the matrix cores.  A is M x K
// (lda), op(B) is K x N: transb == 0 -> B is K x N (ldb), transb != 0 -> B is
// N x K (ldb).  lower_only != 0 leaves every element above the diagonal of C
// untouched and skips the tiles that hold only such elements (M == N expected).
hipError_t launch_gemm_f32(hipStream_t s, int transb, int lower_only, int64_t M, int64_t N,
                           int64_t K, float alpha, const float* A, int64_t lda, const float* B,
                           int64_t ldb, float beta, float* C, int64_t ldc);

hipError_t launch_syrk256_f32(hipStream_t s, int64_t M, const float* A, int64_t lda, float* C, int64_t ldc);

hipError_t launch_hessian_f16(hipStream_t s, const _Float16* X, int64_t n, int64_t p, int64_t ldx,
                              float* H, int64_t ldh, int accumulate, float* partials);
hipError_t launch_mirror_lower(hipStream_t s, float* H, int64_t n, int64_t ldh, const float* src,
                               int64_t lds, int accumulate);

hipError_t launch_cholesky(hipStream_t s, const float* H, int64_t n, int64_t ldh, int precond,
                           float lambda, float* L, int64_t ldl, int* info_dev);

hipError_t launch_init_codebooks(hipStream_t s, const void* W, int w_is_f16, int64_t m, int64_t n,
                                 int64_t ldw, int nbits, int mode, float* T);

hipError_t launch_convert_f16_f32(hipStream_t s, const _Float16* src, int64_t rows, int64_t cols,
                                  int64_t ld_src, float* dst, int64_t ld_dst);

hipError_t launch_update_S(hipStream_t s, const float* W, int64_t m, int64_t n, int64_t ldw,
                           const float* L, int64_t ldl, const float* T, int nbits, uint8_t* Q,
                           int64_t ldq, float* E, int64_t lde, void* scratch);

// T-update on one scratch region: integer digits of H (once per layer), padded copy of Q, the
// one-hot GEMM with fold epilogue, and the per-row assembly + solve (G = W * H is an input,
// computed once per layer).  From the second sweep of a layer on, launch_t_flips lists the columns
// whose code changed and launch_t_delta brings S_i H S_i^T up to date from them when they are few;
// launch_t_accum and launch_t_delta are both enqueued and decide on the device which of them runs.
hipError_t launch_t_prepare(hipStream_t s, const float* H, int64_t m, int64_t n, int64_t ldh,
                            int nbits, void* scratch, int allow_delta);
// cur = 0 / 1: which of the two padded copies of Q is the current sweep's (the other one holds the
// previous sweep's)
hipError_t launch_t_pad(hipStream_t s, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                        int nbits, void* scratch, int cur);
hipError_t launch_t_flips(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur);
hipError_t launch_t_accum(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur);
hipError_t launch_t_delta(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int cur);
// sweep: index of the alternation (0 for a stand-alone T-update); the choice made in it is logged
hipError_t launch_t_solve(hipStream_t s, const float* G, int64_t ldg, int64_t m, int64_t n,
                          const uint8_t* Q, int64_t ldq, int nbits, int empty_mode, float* T,
                          int32_t* empty_count, void* scratch, int sweep);
// log[3 k .. 3 k + 2] = {1 if sweep k updated S_i H S_i^T from the changed columns, 0 if it summed
// it; the largest number of changed indices in a row; their total} (device to host copy of the log
// kept in scratch; synchronises)
constexpr int kTLogMax = 64;
hipError_t read_t_log(hipStream_t s, int64_t m, int64_t n, int nbits, void* scratch, int* modes_host, int count);

// row_loss[i] = sum_j F_ij * E_ij with E = W - T[Q] written to Ebuf first (launch_residual),
// F = E * H by launch_gemm_split, then launch_rowdot.
hipError_t launch_residual(hipStream_t s, const float* W, int64_t m, int64_t n, int64_t ldw,
                           const float* T, const uint8_t* Q, int64_t ldq, int nbits, float* E,
                           int64_t lde);
hipError_t launch_rowdot(hipStream_t s, const float* F, int64_t ldf, const float* E, int64_t lde,
                         int64_t m, int64_t n, float* row_loss);
hipError_t launch_sum_f64(hipStream_t s, const float* v, int64_t m, double* out_dev);

}  // namespace ganq
