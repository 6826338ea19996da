/*
 * ganq.h - C ABI of the MI355X (gfx950) GANQ per-layer solver.
 *
 * GANQ (arXiv 2501.12956) quantises one linear layer W (m x n, m output
 * channels) to a per-row codebook T (m x 2^N) and an index matrix Q (m x n)
 * by minimising |W X - W~ X|_F^2, W~_ij = T_i[Q_ij] (Eq. (1)), for
 * calibration activations X (n x p).  Algorithm 1 alternates a
 * column-sequential assignment update on the Cholesky factor of H = X X^T
 * with a closed-form per-row least-squares codebook update.
 *
 * Conventions for every call
 *   - Every array pointer is a DEVICE pointer owned by the caller unless the
 *     parameter name ends in _host.  The library never frees or keeps a
 *     caller pointer past the call.
 *   - Matrices are row-major with an explicit leading dimension in elements.
 *   - Work is enqueued on the context's HIP stream (ganq_quantize_layer may
 *     also use one internal stream, ordered after the context's stream at entry
 *     and joined before it returns).  Calls that return a host
 *     scalar (info_host, loss_host, loss_history_host) synchronise that
 *     stream before returning; all others are asynchronous.
 *   - Scratch memory comes from a caller-provided workspace
 *     (ganq_workspace_bytes / ganq_set_workspace); the library allocates no
 *     device memory.
 *   - Errors are returned as ganq_status; nothing aborts or throws across the
 *     ABI.  Argument checks run on the host before any GPU work.
 *   - m and n up to 65535; the S-update (and so ganq_quantize_layer) further
 *     needs n * ldl * 4 bytes of L below 4 GiB, i.e. n <= 32767 for a packed L.
 *     Larger shapes return GANQ_ERR_UNSUPPORTED.
 *   - nbits in [1, 4]; C = 2^nbits codes per row.  3 and 4 are the paper's
 *     settings (Section 4.1), 1 and 2 exist for brute-force tests.
 */
#ifndef GANQ_H
#define GANQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ganq_ctx ganq_ctx; /* opaque: one HIP device + one stream + workspace */

/* The enumerations below cross the boundary as plain ints (the C rule).  A C++ translation unit
 * gives them int as their fixed underlying type, so that an out-of-range value handed over by a C
 * caller is a value the library can look at and reject rather than undefined behaviour. */
#ifdef __cplusplus
#define GANQ_ENUM enum : int
#else
#define GANQ_ENUM enum
#endif

typedef GANQ_ENUM {
  GANQ_OK = 0,
  GANQ_ERR_INVALID_ARG = 1,
  GANQ_ERR_UNSUPPORTED = 2,
  GANQ_ERR_NOT_PD = 3,     /* a Cholesky pivot was not finite or not above its threshold (ganq_cholesky) */
  GANQ_ERR_WORKSPACE = 4,  /* workspace missing or too small */
  GANQ_ERR_HIP = 5         /* HIP runtime failure; text in ganq_last_error */
} ganq_status;

typedef GANQ_ENUM { GANQ_F16 = 0, GANQ_F32 = 1 } ganq_dtype;

/* Which matrix is factorised (Eq. (10), Remark 3.1, Appendix A Eq. (23)-(24)). */
typedef GANQ_ENUM {
  GANQ_PRECOND_NONE = 0,    /* H */
  GANQ_PRECOND_LAMBDA = 1,  /* H + lambda I */
  GANQ_PRECOND_DIAGDOM = 2, /* H + Diag(delta), delta_i = max(sum_j|H_ij| - 2 H_ii, 1e-8) */
  GANQ_PRECOND_AUTO = 3     /* NONE, and DIAGDOM if a pivot fails */
} ganq_precond;

/* Rule for the initial codebook T^0 (an input of Algorithm 1 the paper leaves open). */
typedef GANQ_ENUM {
  GANQ_INIT_QUANTILE_MID = 0,       /* level s at row quantile (s + 1/2)/C, linear interpolation */
  GANQ_INIT_QUANTILE_ENDPOINTS = 1, /* level s at row quantile s/(C - 1) */
  GANQ_INIT_MINMAX_GRID = 2         /* C equally spaced values from row min to row max */
} ganq_init;

/* Value given to a code that no column of the row uses (Eq. (7), pseudo-inverse). */
typedef GANQ_ENUM {
  GANQ_EMPTY_ZERO = 0, /* 0, the literal Moore-Penrose result */
  GANQ_EMPTY_KEEP = 1  /* keep the previous codebook entry */
} ganq_empty;

typedef struct {
  ganq_precond precond; /* used when ganq_quantize_layer factors H itself */
  float lambda;         /* for GANQ_PRECOND_LAMBDA */
  ganq_init init;       /* used when init_codebooks != 0 */
  int init_codebooks;   /* 0: T holds T^0 on entry; 1: build T^0 from W */
  ganq_empty empty;
  int flags;            /* 0, or GANQ_OPT_FULL_T_UPDATE; other bits must be 0 */
} ganq_options;

/* ganq_options.flags: sum S_i H S_i^T again in every sweep.  By default a sweep that changed few
 * indices (at most 1 in 24 of them, and at most about n / 2 - between 256 and 16384 - in any row) brings the
 * matrices of the previous sweep up to date from the changed columns instead - the same sums in
 * another order, kept in float64, so T^K may differ from the always-summing path in the last bits
 * of fp32 (and so may a near-tie of a later S-update). */
#define GANQ_OPT_FULL_T_UPDATE 1

/* ---- context ------------------------------------------------------------ */

/* Creates a context bound to HIP device `device` and to `hip_stream`
 * (a hipStream_t, NULL = the default stream).  Touches no GPU state until the
 * first compute call.  *out is set to NULL on failure. */
ganq_status ganq_create(ganq_ctx** out, int device, void* hip_stream);
ganq_status ganq_destroy(ganq_ctx* ctx);

/* Bytes of workspace that any call on a layer of this shape may need
 * (p_tokens = 0 when ganq_build_hessian is not used).  0 on invalid input and for
 * shapes beyond what the calls accept (m or n above 65535, more than 2^40 tokens). */
size_t ganq_workspace_bytes(int64_t m, int64_t n, int64_t p_tokens, int nbits);

/* Hands the context a caller-owned device buffer (256-byte aligned).  It must
 * stay valid until replaced or the context is destroyed. */
ganq_status ganq_set_workspace(ganq_ctx* ctx, void* dev_ptr, size_t bytes);

const char* ganq_status_string(ganq_status s);
/* Text of the last error on this context ("" if none); valid until the next call. */
const char* ganq_last_error(const ganq_ctx* ctx);

/* ---- the seven calls of the hot path ---------------------------------------- */

/* H = X X^T (Algorithm 1; Eq. (9)).  X is n x p (features x tokens) with
 * leading dimension ldx >= p, fp16 or fp32 storage (fp16 products are exact in
 * the fp32 accumulator; fp32 input takes fp32 matrix-core products, nothing is
 * rounded down).  H is n x n fp32,
 * both triangles written.  accumulate != 0 adds to the H already there
 * (streaming token chunks).  Requires p % 8 == 0 and ldx % 8 == 0 for fp16. */
ganq_status ganq_build_hessian(ganq_ctx* ctx, const void* X, ganq_dtype x_dtype, int64_t n,
                               int64_t p, int64_t ldx, float* H, int64_t ldh, int accumulate);

/* The same H = X X^T for activations stored the way calibration batches arrive
 * (Section 4.1 Setup: sequences of tokens through the layer): Xt is p x n
 * (tokens x features) row-major with leading dimension ldxt >= n, so
 * H = Xt^T Xt.  Any p >= 0 and any ldxt >= n.  fp16 activations with
 * n % 8 == 0, ldxt % 8 == 0 and a 16-byte aligned Xt are read in place by the
 * product (LDS transpose reads; the result equals ganq_build_hessian on the
 * transposed array bit for bit).  Anything else is transposed into workspace
 * in chunks (at most 32768 tokens at a time unless the workspace holds more,
 * zero-padded to a multiple of 8) and then takes the path of
 * ganq_build_hessian; accumulate as there. */
ganq_status ganq_build_hessian_tokens(ganq_ctx* ctx, const void* Xt, ganq_dtype x_dtype, int64_t n,
                                      int64_t p, int64_t ldxt, float* H, int64_t ldh,
                                      int accumulate);

/* L = lower Cholesky factor of H (or of its preconditioned form), Eq. (10),
 * Remark 3.1, Appendix A.  L is n x n fp32 with the strict upper triangle
 * zeroed; L may not alias H.  *info_host (optional, may be NULL): 0 on success, k > 0 if pivot k
 * (1-based) was not finite or not above 8 sqrt(n) 2^-24 times the diagonal entry
 * of its column in the matrix being factorised (status GANQ_ERR_NOT_PD; L is
 * then unspecified).  The threshold is the size of the rounding noise of an fp32
 * Schur complement: a pivot below it says the matrix is singular to working
 * precision (fewer tokens than features, duplicated features), which a float64
 * factorisation of the same numbers may not notice; Remark 3.1 / Appendix A are
 * the remedy.  Under GANQ_PRECOND_AUTO a failed plain attempt is repeated with
 * DIAGDOM and *info_host reports the second attempt.  Synchronises. */
ganq_status ganq_cholesky(ganq_ctx* ctx, const float* H, int64_t n, int64_t ldh,
                          ganq_precond precond, float lambda, float* L, int64_t ldl,
                          int64_t* info_host);

/* T^0 from per-row quantiles of W (input of Algorithm 1).  T is m x 2^nbits
 * fp32 row-major, ascending within each row. */
ganq_status ganq_init_codebooks(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                int64_t n, int64_t ldw, int nbits, ganq_init init, float* T);

/* S-update, Eq. (13)-(22) and the inner loop of Algorithm 1: for j = n-1..0
 * and every row i, Q_ij = argmin_s |W_ij + (sum_{u>j} r_iu L_uj)/L_jj - T_is|
 * with r_iu = W_iu - T_i[Q_iu]; ties go to the lowest s.  W m x n fp32,
 * L n x n fp32 lower triangular with positive diagonal, T m x 2^nbits fp32,
 * Q m x n uint8 (one index per byte).  E (optional, may be NULL) receives the
 * residuals W - T[Q], m x n fp32 with leading dimension lde. */
ganq_status ganq_update_S(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                          const float* L, int64_t ldl, const float* T, int nbits, uint8_t* Q,
                          int64_t ldq, float* E, int64_t lde);

/* T-update, Eq. (4)-(7): T_i = W_i H S_i^T (S_i H S_i^T)^dagger for every
 * row, S_i the one-hot form of Q_i.  H is the raw X X^T (n x n fp32,
 * symmetric; both triangles are read).  T holds T^k on entry (used only by
 * GANQ_EMPTY_KEEP) and T^{k+1} on return.  empty_count (optional, m int32)
 * receives the number of unused or numerically dependent codes per row.
 * The off-diagonal entries of H enter S_i H S_i^T as integers of 16, 24 or
 * 32 bits, scaled per row and per column by powers of two and summed
 * exactly; the width is the smallest for which one unit is at most
 * 2^-19 sqrt(H_jj H_kk) (features more than 2^18 below the largest one are
 * measured against that floor).  The diagonal and W H are taken in fp32 and
 * the solve runs in float64. */
ganq_status ganq_update_T(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                          const float* H, int64_t ldh, const uint8_t* Q, int64_t ldq, int nbits,
                          ganq_empty empty, float* T, int32_t* empty_count);

/* Optional: the per-layer inputs of ganq_update_T that do not depend on Q - G = W H and the
 * integer digits of H - computed once and kept at the start of the workspace, so that a caller who
 * drives the alternation of Algorithm 1 itself pays for them once per layer and not once per sweep.
 * Later ganq_update_T calls on this context with the same W, ldw, H, ldh, m, n, nbits use them; any
 * other arguments are served as without this call.  The other calls of this header keep the
 * prepared inputs intact (their scratch goes behind them; ganq_workspace_bytes leaves room) except
 * ganq_quantize_layer, ganq_build_hessian_tokens and ganq_set_workspace, which drop them.  The
 * library does not watch W or H: after changing their contents, call this again.  W == NULL and
 * H == NULL drops what was prepared.  Asynchronous on the context's stream. */
ganq_status ganq_update_T_prepare(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                  const float* H, int64_t ldh, int nbits);

/* Objective of Eq. (1) in the form of Eq. (9): sum_i E_i H E_i^T with
 * E = W - T[Q].  *loss_host receives the total (float64 reduction of fp32
 * row values); row_loss (optional, m fp32, device) the per-row values.
 * Synchronises. */
ganq_status ganq_layer_loss(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                            const float* H, int64_t ldh, const float* T, const uint8_t* Q,
                            int64_t ldq, int nbits, double* loss_host, float* row_loss);

/* Algorithm 1 given H: optional factorisation (L == NULL: factor H here with
 * opts->precond), optional T^0 (opts->init_codebooks), then `iters`
 * alternations of S-update and T-update.  W is m x n fp16 or fp32.  On
 * return T = T^K and Q = Q^K (Q^K was chosen against T^{K-1}; T^K is refit to
 * it).  loss_history_host (optional, 2*iters doubles) receives the objective
 * after every half step (index 2k: after the S-step of sweep k, 2k+1: after
 * its T-step); passing it adds one m x n x n product per half step.
 * opts == NULL means {NONE, 0, QUANTILE_MID, 0, ZERO, 0}.  With L == NULL the work
 * that does not depend on the factor (conversion of W, T^0, G = W H) runs on a
 * second stream of the context beside the factorisation and is joined before
 * the first sweep.  Synchronises. */
ganq_status ganq_quantize_layer(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                int64_t n, int64_t ldw, const float* H, int64_t ldh,
                                const float* L, int64_t ldl, int nbits, int iters,
                                const ganq_options* opts, float* T, uint8_t* Q, int64_t ldq,
                                double* loss_history_host);

/* ---- optional pre-step ------------------------------------------------------ */

/* Outlier split W = W_sparse + W_dense (Appendix B, Algorithm 2; Section 3.3).
 * With p = 1 - r/2, per row the cut-offs are the values at sorted positions
 * lower = ceil(n (1 - p)) and upper = min(floor(n p), n - 1), evaluated as the
 * real-number expressions ceil(n r / 2) and floor(n - n r / 2) (n r / 2 within
 * 1e-9 relative of an integer counts as that integer, so n = 2000, r = 0.01
 * cuts at positions 10 and 1990); entries >= the upper or <= the lower cut-off
 * are outliers.  W is m x n fp16 or fp32; W_dense is m x n fp32 with zeros at
 * the outlier positions and feeds ganq_quantize_layer unchanged.  W_sparse is
 * returned as CSR: row_ptr (m + 1 entries, int64), col_idx and values (columns
 * ascending within a row; values are the stored weights, exact).  capacity =
 * entries that col_idx / values can hold; *nnz_host receives the number of
 * outliers.  If it exceeds capacity the status is GANQ_ERR_INVALID_ARG,
 * W_dense and row_ptr are complete and the first `capacity` entries were
 * written: call again with larger arrays.  0 <= r < 1; n <= 32768.
 * Synchronises. */
ganq_status ganq_outlier_split(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m, int64_t n,
                               int64_t ldw, double r, float* W_dense, int64_t ldd, int64_t* row_ptr,
                               int32_t* col_idx, float* values, int64_t capacity, int64_t* nnz_host);

/* ganq_outlier_split for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same kernels, same results, but the per-row scratch (two cut-off values and one
 * count per row, 12 bytes a row) lives in an array that is part of the library's device image,
 * 768 KiB per GPU for the life of the process, sized for m <= 65536 rows.  More rows return
 * GANQ_ERR_UNSUPPORTED.  The call needs no ganq_set_workspace, allocates nothing (no hipMalloc,
 * hipFree, events or streams) and takes no timing brackets.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (from different contexts or streams) race
 * and must be serialised by the caller.  Nothing in the array has to survive or be cleared
 * between calls: every entry a call reads it has written itself.  Synchronises. */
ganq_status ganq_outlier_split_noalloc(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                       int64_t n, int64_t ldw, double r, float* W_dense, int64_t ldd,
                                       int64_t* row_ptr, int32_t* col_idx, float* values,
                                       int64_t capacity, int64_t* nnz_host);

/* ---- deployment: stored form and look-up-table product ---------------------- */

/* Stored form of a quantized layer (Table 1): per row the n N-bit codes and a
 * table of 2^N fp16 values (0.5 m n + 32 m bytes at 4 bits when n is a multiple
 * of 32).  Codes: row i starts at packed + i * ldp bytes and is a little-endian
 * bit stream, code j in bits [N j, N j + N), bit b of the stream being bit
 * (b mod 8) of byte b / 8; unused bits up to ganq_packed_row_bytes() are zero.
 * ganq_packed_row_bytes = 4 N ceil(n / 32), rounded up to a multiple of 16
 * (0 for n <= 0, n > 2^40 or N outside 1..4). */
int64_t ganq_packed_row_bytes(int64_t n, int nbits);

/* Q (m x n codes, device) and T (m x 2^N fp32, device) -> packed (m rows of ldp
 * bytes, device, 16-byte aligned, ldp % 16 == 0, ldp >= ganq_packed_row_bytes)
 * and lut (m x 2^N IEEE binary16 bit patterns, device; T rounded to nearest
 * even).  1 <= nbits <= 4, m <= 65535.  Asynchronous on the context's stream. */
ganq_status ganq_pack_layer(ganq_ctx* ctx, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                            const float* T, int nbits, uint8_t* packed, int64_t ldp, uint16_t* lut);

/* y = W~ x (+ W_sparse x), W~_ij = lut_i[Q_ij]: the look-up-table product of
 * Figure 1(a) for one activation vector (batch-1 decoding, Section 4.4), with
 * the sparse part of GANQ* (Section 3.3) when row_ptr != NULL.  packed / ldp /
 * lut as written by ganq_pack_layer; x: n fp16 values (device); y: m fp32
 * (device); row_ptr (m + 1, int64), col_idx (int32, each < n) and values (fp32)
 * are the CSR arrays of ganq_outlier_split (device) or all NULL.  fp16 x fp16
 * products, fp32 accumulation; the result is bit-reproducible.  Asynchronous on
 * the context's stream; uses no workspace. */
ganq_status ganq_lut_gemv(ganq_ctx* ctx, const uint8_t* packed, int64_t ldp, const uint16_t* lut,
                          int nbits, int64_t m, int64_t n, const void* x, float* y,
                          const int64_t* row_ptr, const int32_t* col_idx, const float* values);

/* ---- optional per-kernel timing (measurement aid, not part of the method) ------ */

/* Kernel classes the library launches; one step of Algorithm 1 touches all of them. */
typedef GANQ_ENUM {
  GANQ_K_HESSIAN = 0,  /* H = X X^T product (+ partial-sum reduction) */
  GANQ_K_CHOLESKY = 1, /* whole blocked factorisation */
  GANQ_K_INIT = 2,     /* T^0 (and fp16 -> fp32 conversion of W) */
  GANQ_K_GEMM_WH = 3,  /* G = W H, once per layer */
  GANQ_K_UPDATE_S = 4, /* one S-update sweep (one launch) */
  GANQ_K_T_PREP = 5,   /* integer digits of H for the T-update, once per layer */
  GANQ_K_T_PAD = 6,    /* padded copy of Q (and the list of changed columns), once per sweep */
  GANQ_K_T_ACCUM = 7,  /* one-hot GEMM of the T-update, once per sweep */
  GANQ_K_T_SOLVE = 8,  /* per-row assembly and solve, once per sweep */
  GANQ_K_LOSS = 9,     /* objective evaluation */
  GANQ_K_OUTLIER = 10, /* outlier split (sort, offsets, compaction) */
  GANQ_K_PACK = 11,    /* stored form: bit packing and fp16 tables */
  GANQ_K_LUT_GEMV = 12,/* look-up-table product for one activation vector */
  GANQ_K_T_DELTA = 13, /* update of S_i H S_i^T from the changed columns, in sweeps with few changes */
  GANQ_K_T_SKIP = 14,  /* launches of T_ACCUM / T_DELTA that found the other one chosen and returned */
  GANQ_K_COUNT = 15
} ganq_kernel_class;

/* on != 0: bracket every kernel class launched through this context with HIP
 * events on the context's stream and accumulate the elapsed time; resets the
 * accumulated figures.  on == 0: stop. */
ganq_status ganq_profile_enable(ganq_ctx* ctx, int on);
/* Synchronises the stream, then writes the accumulated milliseconds and number
 * of bracketed launches per class (arrays of GANQ_K_COUNT, host memory). */
ganq_status ganq_profile_read(ganq_ctx* ctx, double* ms_host, int64_t* launches_host);

/* What the sweeps of the last ganq_quantize_layer call on this context did (host memory only, no
 * GPU work): *sweeps_host = number of logged sweeps (at most 64; 0 if the call ran with
 * GANQ_OPT_FULL_T_UPDATE or a single sweep), and for sweep k < min(*sweeps_host, capacity):
 * log_host[3k] = 1 if it updated S_i H S_i^T from the changed columns, 0 if it summed it again;
 * log_host[3k+1] = the largest number of indices that changed in one row against the sweep
 * before; log_host[3k+2] = their total (both 0 for the first sweep).  log_host may be NULL;
 * capacity >= 0. */
ganq_status ganq_sweep_log(const ganq_ctx* ctx, int32_t* log_host, int capacity, int* sweeps_host);

/* Rates this GPU sustains on bare loops, for roofline fractions against measured rather than
 * published peaks: peaks_host[0] = fp16 matrix-core TFLOP/s (v_mfma_f32_32x32x16_f16),
 * [1] = fp32 matrix-core TFLOP/s (v_mfma_f32_32x32x2_f32), [2] = int8 matrix-core TOP/s
 * (v_mfma_i32_32x32x32_i8), each from a register-resident loop with four independent
 * accumulators per wavefront and two wavefronts per SIMD; [3] = GB/s (read + write) of a plain
 * device copy of half the workspace (at most 1 GiB).  Best of three timed launches each, HIP
 * events on the context's stream.  Needs a workspace of at least 2 MiB.  Synchronises. */
ganq_status ganq_measure_peaks(ganq_ctx* ctx, double* peaks_host /* 4 */);

#ifdef __cplusplus
}
#endif
#endif /* GANQ_H */
