/* Calls every entry point of ganq.h with arguments that the host-side validation must reject (or
 * accept without GPU work), from a plain C program.  Built against a copy of the library whose
 * host code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer and run on a
 * machine without a GPU: any out-of-bounds access, misaligned access, signed overflow or shift
 * error in the argument checking aborts the run.  The device pointers are made-up addresses:
 * a check that dereferenced one would be reported as well.  Exit status 0 = every call returned
 * what the header promises. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "ganq.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
  do {                                                                                  \
    const long long got_ = (long long)(call);                                           \
    if (got_ != (long long)(want)) {                                                    \
      fprintf(stderr, "line %d: %s returned %lld, expected %lld\n", __LINE__, #call, got_, \
              (long long)(want));                                                       \
      ++failures;                                                                       \
    }                                                                                   \
  } while (0)

int main(void) {
  void* const fake = (void*)(uintptr_t)0x1000;
  void* const fake2 = (void*)(uintptr_t)0x2000;
  void* const odd = (void*)(uintptr_t)0x1004;
  const ganq_status inv = GANQ_ERR_INVALID_ARG, uns = GANQ_ERR_UNSUPPORTED;
  ganq_ctx* h = NULL;
  int64_t info = 7, nnz = -1;
  double loss = 1.0;

  EXPECT(ganq_create(NULL, 0, NULL), inv);
  EXPECT(ganq_create(&h, -1, NULL), inv);
  EXPECT(ganq_create(&h, 0, NULL), GANQ_OK);
  if (h == NULL) { fprintf(stderr, "no context\n"); return 2; }

  /* status strings and size queries, including extreme arguments */
  for (int s = -3; s < 12; ++s) EXPECT(ganq_status_string((ganq_status)s) == NULL, 0);
  EXPECT(ganq_workspace_bytes(0, 0, 0, 4), 0);
  EXPECT(ganq_workspace_bytes(16, 64, 0, 5), 0);
  EXPECT(ganq_workspace_bytes(-1, 64, 0, 4), 0);
  EXPECT(ganq_workspace_bytes(4096, 4096, 262144, 4) > 0, 1);
  EXPECT(ganq_workspace_bytes(65535, 32768, INT64_MAX / 4, 4) >= 0, 1);
  EXPECT(ganq_workspace_bytes(INT64_MAX, INT64_MAX, INT64_MAX, 4) >= 0, 1);
  EXPECT(ganq_packed_row_bytes(4096, 4), 2048);
  EXPECT(ganq_packed_row_bytes(33, 3), 32);
  EXPECT(ganq_packed_row_bytes(0, 4), 0);
  EXPECT(ganq_packed_row_bytes(8, 5), 0);
  EXPECT(ganq_packed_row_bytes(-5, 4), 0);
  EXPECT(ganq_packed_row_bytes(INT64_MAX, 4) >= 0, 1);

  /* null context on every call that takes one */
  EXPECT(ganq_destroy(NULL), inv);
  EXPECT(ganq_set_workspace(NULL, NULL, 0), inv);
  EXPECT(ganq_last_error(NULL) == NULL, 0);
  EXPECT(ganq_build_hessian(NULL, fake, GANQ_F16, 8, 8, 8, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian_tokens(NULL, fake, GANQ_F16, 8, 8, 8, fake, 8, 0), inv);
  EXPECT(ganq_cholesky(NULL, fake, 8, 8, GANQ_PRECOND_NONE, 0.f, fake2, 8, &info), inv);
  EXPECT(ganq_init_codebooks(NULL, fake, GANQ_F32, 4, 8, 8, 4, GANQ_INIT_QUANTILE_MID, fake), inv);
  EXPECT(ganq_update_S(NULL, fake, 1, 1, 1, fake, 1, fake, 4, fake, 1, NULL, 0), inv);
  EXPECT(ganq_update_T(NULL, fake, 4, 8, 8, fake, 8, fake, 8, 4, GANQ_EMPTY_ZERO, fake, NULL), inv);
  EXPECT(ganq_update_T_prepare(NULL, fake, 4, 8, 8, fake, 8, 4), inv);
  EXPECT(ganq_layer_loss(NULL, fake, 4, 8, 8, fake, 8, fake, fake, 8, 4, &loss, NULL), inv);
  EXPECT(ganq_quantize_layer(NULL, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 4, 1, NULL, fake, fake, 8, NULL), inv);
  EXPECT(ganq_outlier_split(NULL, fake, GANQ_F32, 4, 8, 8, 0.1, fake, 8, fake, fake, fake, 8, &nnz), inv);
  EXPECT(ganq_outlier_split_noalloc(NULL, fake, GANQ_F32, 4, 8, 8, 0.1, fake, 8, fake, fake, fake, 8, &nnz), inv);
  EXPECT(ganq_pack_layer(NULL, fake, 4, 64, 64, fake, 4, fake, 32, fake), inv);
  EXPECT(ganq_lut_gemv(NULL, fake, 32, fake, 4, 4, 64, fake, fake, NULL, NULL, NULL), inv);
  EXPECT(ganq_profile_enable(NULL, 1), inv);
  EXPECT(ganq_profile_read(NULL, NULL, NULL), inv);
  EXPECT(ganq_sweep_log(NULL, NULL, 0, NULL), inv);
  EXPECT(ganq_measure_peaks(NULL, NULL), inv);

  /* bad sizes, leading dimensions, widths, enums, aliasing */
  EXPECT(ganq_build_hessian(h, fake, GANQ_F16, 0, 8, 8, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian(h, fake, GANQ_F16, 8, 16, 8, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian(h, fake, (ganq_dtype)7, 8, 16, 16, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian(h, fake, GANQ_F16, 8, 16, 20, fake, 8, 0), uns);
  EXPECT(ganq_build_hessian(h, fake, GANQ_F16, 8, 16, 16, fake, 4, 0), inv);
  EXPECT(ganq_build_hessian(h, NULL, GANQ_F16, 8, 16, 16, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian(h, fake, GANQ_F16, INT64_MAX, 16, 16, fake, INT64_MAX, 0) != GANQ_OK, 1);
  EXPECT(ganq_build_hessian_tokens(h, fake, GANQ_F16, 8, 16, 4, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian_tokens(h, fake, GANQ_F16, 8, -1, 8, fake, 8, 0), inv);
  EXPECT(ganq_build_hessian_tokens(h, fake, (ganq_dtype)-1, 8, 16, 8, fake, 8, 0), inv);
  EXPECT(ganq_cholesky(h, fake, 8, 4, GANQ_PRECOND_NONE, 0.f, fake2, 8, &info), inv);
  EXPECT(info, 0);
  EXPECT(ganq_cholesky(h, fake, 8, 8, GANQ_PRECOND_NONE, 0.f, fake, 8, &info), inv);
  EXPECT(ganq_cholesky(h, fake, 8, 8, GANQ_PRECOND_LAMBDA, 0.f, fake2, 8, &info), inv);
  EXPECT(ganq_cholesky(h, fake, 8, 8, (ganq_precond)9, 0.f, fake2, 8, &info), inv);
  EXPECT(ganq_cholesky(h, fake, 8, 8, GANQ_PRECOND_NONE, 0.f, NULL, 8, NULL), inv);
  EXPECT(ganq_cholesky(h, fake, 70000, 70000, GANQ_PRECOND_NONE, 0.f, fake2, 70000, NULL), uns);
  EXPECT(ganq_init_codebooks(h, fake, GANQ_F32, 4, 8, 8, 0, GANQ_INIT_QUANTILE_MID, fake), inv);
  EXPECT(ganq_init_codebooks(h, fake, GANQ_F32, 4, 8, 8, 5, GANQ_INIT_QUANTILE_MID, fake), inv);
  EXPECT(ganq_init_codebooks(h, fake, GANQ_F32, 4, 8, 8, 4, (ganq_init)3, fake), inv);
  EXPECT(ganq_init_codebooks(h, fake, GANQ_F32, 4, 40000, 40000, 4, GANQ_INIT_QUANTILE_MID, fake), uns);
  EXPECT(ganq_update_S(h, fake, 4, 8, 7, fake, 8, fake, 4, fake, 8, NULL, 0), inv);
  EXPECT(ganq_update_S(h, fake, 4, 8, 8, NULL, 8, fake, 4, fake, 8, NULL, 0), inv);
  EXPECT(ganq_update_S(h, fake, 4, 8, 8, fake, 8, fake, 4, fake, 8, fake, 4), inv);
  EXPECT(ganq_update_S(h, fake, 4, 8, 8, fake, 8, fake, 9, fake, 8, NULL, 0), inv);
  EXPECT(ganq_update_S(h, fake, 4, 40000, 40000, fake, 40000, fake, 4, fake, 40000, NULL, 0), uns);
  EXPECT(ganq_update_T(h, fake, 4, 8, 8, fake, 8, fake, 8, 4, (ganq_empty)2, fake, NULL), inv);
  EXPECT(ganq_update_T(h, fake, 4, 8, 8, fake, 8, NULL, 8, 4, GANQ_EMPTY_ZERO, fake, NULL), inv);
  EXPECT(ganq_update_T(h, fake, 4, 8, 8, fake, 4, fake, 8, 4, GANQ_EMPTY_ZERO, fake, NULL), inv);
  EXPECT(ganq_update_T_prepare(h, fake, 4, 8, 4, fake, 8, 4), inv);
  EXPECT(ganq_update_T_prepare(h, fake, 4, 8, 8, NULL, 8, 4), inv);
  EXPECT(ganq_update_T_prepare(h, NULL, 0, 0, 0, NULL, 0, 0), GANQ_OK);
  EXPECT(ganq_layer_loss(h, fake, 4, 8, 8, fake, 8, fake, fake, 8, 4, NULL, NULL), inv);
  EXPECT(ganq_layer_loss(h, fake, 4, -1, 8, fake, 8, fake, fake, 8, 4, &loss, NULL), inv);
  {
    ganq_options o;
    memset(&o, 0, sizeof o);
    o.flags = 2;
    EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 4, 1, &o, fake, fake, 8, NULL), inv);
    o.flags = 0;
    o.precond = (ganq_precond)11;
    EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 4, 1, &o, fake, fake, 8, NULL), inv);
    o.precond = GANQ_PRECOND_NONE;
    o.empty = (ganq_empty)5;
    EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 4, 1, &o, fake, fake, 8, NULL), inv);
  }
  EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 4, -1, NULL, fake, fake, 8, NULL), inv);
  EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 8, fake, 8, NULL, 0, 0, 1, NULL, fake, fake, 8, NULL), inv);
  EXPECT(ganq_quantize_layer(h, fake, GANQ_F32, 4, 8, 4, fake, 8, NULL, 0, 4, 1, NULL, fake, fake, 8, NULL), inv);
  EXPECT(ganq_outlier_split(h, fake, GANQ_F32, 4, 8, 8, 1.0, fake, 8, fake, fake, fake, 8, &nnz), inv);
  EXPECT(ganq_outlier_split(h, fake, GANQ_F32, 4, 8, 8, -0.1, fake, 8, fake, fake, fake, 8, &nnz), inv);
  EXPECT(ganq_outlier_split(h, fake, GANQ_F32, 4, 8, 8, 0.1, fake, 8, fake, fake, fake, 8, NULL), inv);
  EXPECT(ganq_outlier_split(h, fake, GANQ_F32, 4, 40000, 40000, 0.1, fake, 40000, fake, fake, fake, 8, &nnz), uns);
  EXPECT(ganq_outlier_split_noalloc(h, fake, GANQ_F32, 70000, 8, 8, 0.1, fake, 8, fake, fake, fake, 8, &nnz), uns);
  EXPECT(ganq_outlier_split_noalloc(h, fake, GANQ_F32, 4, 8, 4, 0.1, fake, 8, fake, fake, fake, 8, &nnz), inv);
  EXPECT(ganq_pack_layer(h, fake, 4, 64, 64, fake, 5, fake, 32, fake), inv);
  EXPECT(ganq_pack_layer(h, fake, 4, 64, 32, fake, 4, fake, 32, fake), inv);
  EXPECT(ganq_pack_layer(h, fake, 4, 64, 64, fake, 4, fake, 16, fake), inv);
  EXPECT(ganq_pack_layer(h, fake, 4, 64, 64, fake, 4, odd, 32, fake), inv);
  EXPECT(ganq_pack_layer(h, fake, 70000, 64, 64, fake, 4, fake, 32, fake), uns);
  EXPECT(ganq_lut_gemv(h, fake, 24, fake, 4, 4, 64, fake, fake, NULL, NULL, NULL), inv);
  EXPECT(ganq_lut_gemv(h, fake, 32, fake, 0, 4, 64, fake, fake, NULL, NULL, NULL), inv);
  EXPECT(ganq_lut_gemv(h, fake, 32, fake, 4, 4, 64, NULL, fake, NULL, NULL, NULL), inv);
  EXPECT(ganq_lut_gemv(h, fake, 32, fake, 4, 4, 64, fake, fake, fake, NULL, NULL), inv);
  EXPECT(ganq_last_error(h) != NULL && ganq_last_error(h)[0] != 0, 1);

  /* empty problems are accepted without GPU work */
  EXPECT(ganq_update_S(h, NULL, 0, 8, 8, fake, 8, NULL, 4, NULL, 8, NULL, 0), GANQ_OK);
  EXPECT(ganq_layer_loss(h, NULL, 0, 8, 8, fake, 8, NULL, NULL, 8, 4, &loss, NULL), GANQ_OK);
  EXPECT(loss == 0.0, 1);

  /* host-only calls */
  {
    int32_t log[9];
    int sweeps = -1;
    EXPECT(ganq_sweep_log(h, log, 3, &sweeps), GANQ_OK);
    EXPECT(sweeps, 0);
    EXPECT(ganq_sweep_log(h, NULL, 0, &sweeps), GANQ_OK);
    EXPECT(ganq_sweep_log(h, log, -1, &sweeps), inv);
    EXPECT(ganq_sweep_log(h, log, 3, NULL), inv);
  }
  EXPECT(ganq_set_workspace(h, (void*)(uintptr_t)0x1001, 64), inv);
  EXPECT(ganq_set_workspace(h, NULL, 64), inv);
  EXPECT(ganq_set_workspace(h, NULL, 0), GANQ_OK);
  EXPECT(ganq_measure_peaks(h, NULL), inv);
  EXPECT(ganq_destroy(h), GANQ_OK);

  if (failures) {
    fprintf(stderr, "%d unexpected results\n", failures);
    return 1;
  }
  printf("abi sanitize driver: all calls returned as documented\n");
  return 0;
}
