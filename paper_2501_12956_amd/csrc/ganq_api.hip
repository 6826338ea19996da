// Host side of the C ABI declared in ganq.h: argument checks, workspace
// carving, and the order in which the gfx950 kernels are enqueued.  No
// arithmetic of the method lives here.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "ganq_internal.h"

using namespace ganq;

namespace {

ganq_status fail(ganq_ctx* ctx, ganq_status st, const char* msg) {
  if (ctx != nullptr) ctx->last_error = msg;
  return st;
}

ganq_status hip_fail(ganq_ctx* ctx, hipError_t e, const char* where) {
  if (ctx != nullptr) {
    ctx->last_error = std::string(where) + ": " + hipGetErrorString(e);
  }
  return GANQ_ERR_HIP;
}

#define GANQ_HIP(ctx, expr)                                     \
  do {                                                          \
    hipError_t _e = (expr);                                     \
    if (_e != hipSuccess) return hip_fail((ctx), _e, #expr);    \
  } while (0)

#define GANQ_REQUIRE(ctx, cond, msg)                                      \
  do {                                                                    \
    if (!(cond)) return fail((ctx), GANQ_ERR_INVALID_ARG, (msg));         \
  } while (0)

// ---- per-class event brackets ----
struct ProfScope {
  ganq_ctx* ctx;
  int cls;
  hipStream_t st;
  hipEvent_t a = nullptr, b = nullptr;
  bool live = false;
  static hipEvent_t get(ganq_ctx* c) {
    if (!c->prof_free.empty()) {
      hipEvent_t e = c->prof_free.back();
      c->prof_free.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  // events go on the stream the bracketed kernels are launched on
  int tag = -1;
  ProfScope(ganq_ctx* c, int k, hipStream_t on = nullptr, int tg = -1)
      : ctx(c), cls(k), st(on != nullptr ? on : c->stream), tag(tg) {
    if (!c->prof_on) return;
    a = get(c);
    b = get(c);
    if (a == nullptr || b == nullptr) return;
    live = hipEventRecord(a, st) == hipSuccess;
  }
  ~ProfScope() {
    if (!live) return;
    if (hipEventRecord(b, st) == hipSuccess)
      ctx->prof_pending.push_back({cls, a, b, tag});
    ctx->prof_launches[cls] += 1;
  }
};

void prof_drain(ganq_ctx* ctx) {
  for (auto& r : ctx->prof_pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) ctx->prof_ms[r.cls] += ms;
    ctx->prof_free.push_back(r.a);
    ctx->prof_free.push_back(r.b);
  }
  ctx->prof_pending.clear();
}

bool nbits_ok(int nbits) { return nbits >= 1 && nbits <= 4; }
// several kernels put a matrix dimension on the y axis of the launch grid
constexpr int64_t kMaxDim = 65535;
bool dtype_ok(int d) { return d == GANQ_F16 || d == GANQ_F32; }

ganq_status bind_device(ganq_ctx* ctx) {
  GANQ_HIP(ctx, hipSetDevice(ctx->device));
  ctx->device_ready = true;
  return GANQ_OK;
}

size_t quantize_scratch_bytes(int64_t m, int64_t n, int nbits) {
  size_t b = 0;
  b += align_up((size_t)m * n * sizeof(float));        // W in fp32
  b += align_up((size_t)n * n * sizeof(float));        // L
  b += align_up((size_t)m * n * sizeof(float));        // G = W H
  b += cholesky_scratch_bytes(n);
  b += update_s_scratch_bytes(m, n);
  b += update_t_scratch_bytes(m, n, nbits);
  b += loss_scratch_bytes(m, n);
  b += outlier_scratch_bytes(m);
  b += gemm_split_scratch_bytes(m, n, n);
  return b + 8 * kAlign;
}

// Scratch arena of a stand-alone call: behind the prepared T-update inputs when they are valid and
// `need` bytes still fit there, else from the start of the workspace (which drops the prepared inputs).
Arena call_arena(ganq_ctx* ctx, size_t need) {
  Arena ar(ctx->ws, ctx->ws_bytes);
  if (ctx->tprep.valid) {
    if (ctx->tprep.ws == ctx->ws && align_up(ctx->tprep.bytes) + need + 2 * kAlign <= ctx->ws_bytes)
      ar.off = align_up(ctx->tprep.bytes);
    else
      ctx->tprep.valid = false;
  }
  return ar;
}

// row losses -> host double; scratch = [E][F][row values][double]
ganq_status run_loss(ganq_ctx* ctx, Arena& ar, const float* W, int64_t m, int64_t n, int64_t ldw,
                     const float* H, int64_t ldh, const float* T, const uint8_t* Q, int64_t ldq,
                     int nbits, double* loss_host, float* row_loss_out, void* gs = nullptr) {
  if (gs == nullptr) gs = ar.take(gemm_split_scratch_bytes(m, n, n));
  float* E = (float*)ar.take((size_t)m * n * sizeof(float));
  float* F = (float*)ar.take((size_t)m * n * sizeof(float));
  float* rows = (float*)ar.take((size_t)m * sizeof(float));
  double* total = (double*)ar.take(sizeof(double));
  if (gs == nullptr || E == nullptr || F == nullptr || rows == nullptr || total == nullptr)
    return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for the loss evaluation");
  hipStream_t s = ctx->stream;
  ProfScope prof(ctx, GANQ_K_LOSS);
  GANQ_HIP(ctx, launch_residual(s, W, m, n, ldw, T, Q, ldq, nbits, E, n));
  // F = E H; H is symmetric, so its rows serve as the rows of the right operand
  GANQ_HIP(ctx, launch_gemm_split(s, m, n, n, E, n, H, ldh, F, n, gs, 0));
  float* rl = (row_loss_out != nullptr) ? row_loss_out : rows;
  GANQ_HIP(ctx, launch_rowdot(s, F, n, E, n, m, n, rl));
  GANQ_HIP(ctx, launch_sum_f64(s, rl, m, total));
  GANQ_HIP(ctx, hipMemcpyAsync(loss_host, total, sizeof(double), hipMemcpyDeviceToHost, s));
  GANQ_HIP(ctx, hipStreamSynchronize(s));
  return GANQ_OK;
}

ganq_status run_cholesky(ganq_ctx* ctx, Arena& ar, const float* H, int64_t n, int64_t ldh,
                         int precond, float lambda, float* L, int64_t ldl, int64_t* info_host) {
  int* info_dev = (int*)ar.take(cholesky_scratch_bytes(n));
  if (info_dev == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for Cholesky");
  hipStream_t s = ctx->stream;
  int first = (precond == GANQ_PRECOND_AUTO) ? GANQ_PRECOND_NONE : precond;
  int info = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    const int mode = (attempt == 0) ? first : GANQ_PRECOND_DIAGDOM;
    {
      ProfScope prof(ctx, GANQ_K_CHOLESKY);
      GANQ_HIP(ctx, launch_cholesky(s, H, n, ldh, mode, lambda, L, ldl, info_dev));
    }
    GANQ_HIP(ctx, hipMemcpyAsync(&info, info_dev, sizeof(int), hipMemcpyDeviceToHost, s));
    GANQ_HIP(ctx, hipStreamSynchronize(s));
    if (info == 0 || precond != GANQ_PRECOND_AUTO) break;
  }
  if (info_host != nullptr) *info_host = info;
  if (info != 0) {
    char buf[96];
    snprintf(buf, sizeof buf, "matrix not positive definite at pivot %d", info);
    return fail(ctx, GANQ_ERR_NOT_PD, buf);
  }
  return GANQ_OK;
}

// ---- scratch of the allocation-free outlier split ----
// Per-row cut-off pairs and outlier counts of at most kStaticOutlierRows rows, laid out exactly as
// launch_outlier_split lays out a workspace of that many rows.  Every device the library runs on
// holds its own copy of this array at its own address until the process ends; the name below is
// only a host-side handle, the device address comes from hipGetSymbolAddress once per device.
constexpr int64_t kStaticOutlierRows = 65536;
constexpr size_t kStaticOutlierBytes = 2 * sizeof(float) * kStaticOutlierRows + sizeof(int32_t) * kStaticOutlierRows;
static __device__ __align__(256) unsigned char g_outlier_scratch[kStaticOutlierBytes];
constexpr int kMaxDevices = 64;
std::mutex g_outlier_mu;
void* g_outlier_ptr[kMaxDevices] = {nullptr};

// Device address of this device's copy of the array; the device must be current.
hipError_t static_outlier_scratch(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_outlier_mu);
  if (g_outlier_ptr[device] == nullptr) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_outlier_scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_outlier_ptr[device] = p;
  }
  *out = g_outlier_ptr[device];
  return hipSuccess;
}

// Both outlier-split entry points; they differ only in where the per-row scratch lives.
ganq_status outlier_split_impl(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m, int64_t n,
                               int64_t ldw, double r, float* W_dense, int64_t ldd, int64_t* row_ptr,
                               int32_t* col_idx, float* values, int64_t capacity, int64_t* nnz_host,
                               bool static_scratch) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  if (nnz_host != nullptr) *nnz_host = 0;
  GANQ_REQUIRE(ctx, dtype_ok(w_dtype), "w_dtype");
  GANQ_REQUIRE(ctx, m > 0 && n > 0, "m and n must be positive");
  GANQ_REQUIRE(ctx, W != nullptr && ldw >= n, "W / ldw");
  GANQ_REQUIRE(ctx, W_dense != nullptr && ldd >= n, "W_dense / ldd");
  GANQ_REQUIRE(ctx, row_ptr != nullptr && nnz_host != nullptr, "row_ptr / nnz_host");
  GANQ_REQUIRE(ctx, capacity >= 0 && (capacity == 0 || (col_idx != nullptr && values != nullptr)),
               "col_idx / values / capacity");
  GANQ_REQUIRE(ctx, r >= 0.0 && r < 1.0, "r must be in [0, 1)");
  if (n > 32768) return fail(ctx, GANQ_ERR_UNSUPPORTED, "outlier split sorts a row in LDS: n <= 32768");
  if (static_scratch && (m > kStaticOutlierRows || outlier_scratch_bytes(m) > kStaticOutlierBytes))
    return fail(ctx, GANQ_ERR_UNSUPPORTED,
                "ganq_outlier_split_noalloc holds scratch for at most 65536 rows: split the layer by rows "
                "or use ganq_outlier_split with a workspace");
  // Sorted positions of the two cut-offs: ceil(n (1 - p)) and floor(n p), p = 1 - r/2, taken as
  // real-number expressions of t = n r / 2 (1 - (1 - r/2) is not r/2 in binary floating point).
  // A t that is an integer up to rounding is that integer: n = 2000, r = 0.01 cuts at 10 and 1990.
  double t = (double)n * (0.5 * r);
  const double tn = nearbyint(t);
  if (fabs(t - tn) <= 1e-9 * fmax(1.0, fabs(t))) t = tn;
  int64_t upper = (int64_t)floor((double)n - t);
  if (upper > n - 1) upper = n - 1;
  const int64_t lower = (int64_t)ceil(t);
  GANQ_REQUIRE(ctx, lower >= 0 && lower <= n - 1, "r too large for this n");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  void* scratch = nullptr;
  if (static_scratch) {
    // every entry the kernels read is written earlier in the same call (cut-offs and counts of rows
    // 0..m-1), so nothing left by a previous call has to be cleared
    GANQ_HIP(ctx, static_outlier_scratch(ctx->device, &scratch));
  } else {
    Arena ar = call_arena(ctx, outlier_scratch_bytes(m));
    scratch = ar.take(outlier_scratch_bytes(m));
    if (scratch == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for the outlier split");
  }
  if (static_scratch) {
    // no event brackets here: they may create HIP events
    GANQ_HIP(ctx, launch_outlier_split(s, W, w_dtype == GANQ_F16, m, n, ldw, (int)lower, (int)upper, W_dense,
                                       ldd, row_ptr, col_idx, values, capacity, scratch));
  } else {
    ProfScope prof(ctx, GANQ_K_OUTLIER);
    GANQ_HIP(ctx, launch_outlier_split(s, W, w_dtype == GANQ_F16, m, n, ldw, (int)lower, (int)upper, W_dense,
                                       ldd, row_ptr, col_idx, values, capacity, scratch));
  }
  int64_t nnz = 0;
  GANQ_HIP(ctx, hipMemcpyAsync(&nnz, row_ptr + m, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GANQ_HIP(ctx, hipStreamSynchronize(s));
  *nnz_host = nnz;
  if (nnz > capacity) {
    char buf[128];
    snprintf(buf, sizeof buf, "%lld outliers do not fit a capacity of %lld", (long long)nnz,
             (long long)capacity);
    return fail(ctx, GANQ_ERR_INVALID_ARG, buf);
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

}  // namespace

extern "C" {

ganq_status ganq_create(ganq_ctx** out, int device, void* hip_stream) {
  if (out == nullptr) return GANQ_ERR_INVALID_ARG;
  *out = nullptr;
  if (device < 0) return GANQ_ERR_INVALID_ARG;
  ganq_ctx* c = new (std::nothrow) ganq_ctx();
  if (c == nullptr) return GANQ_ERR_HIP;
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  *out = c;
  return GANQ_OK;
}

ganq_status ganq_destroy(ganq_ctx* ctx) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  for (auto& r : ctx->prof_pending) {
    hipEventDestroy(r.a);
    hipEventDestroy(r.b);
  }
  for (auto e : ctx->prof_free) hipEventDestroy(e);
  if (ctx->fork_ev != nullptr) hipEventDestroy(ctx->fork_ev);
  if (ctx->join_ev != nullptr) hipEventDestroy(ctx->join_ev);
  if (ctx->side != nullptr) hipStreamDestroy(ctx->side);
  delete ctx;
  return GANQ_OK;
}

size_t ganq_workspace_bytes(int64_t m, int64_t n, int64_t p_tokens, int nbits) {
  if (m < 0 || n <= 0 || p_tokens < 0 || !nbits_ok(nbits)) return 0;
  // shapes no call accepts; also keeps every product below within 64 bits
  if (m > kMaxDim || n > kMaxDim || p_tokens > ((int64_t)1 << 40)) return 0;
  size_t q = quantize_scratch_bytes(m, n, nbits);
  size_t h = hessian_scratch_bytes(n, p_tokens > 0 ? p_tokens : 1) + kAlign;
  size_t h32 = align_up((size_t)n * n * sizeof(float)) + kAlign;
  if (h32 > h) h = h32;
  if (p_tokens > 0) {     // token-major entry point: transposed chunk + the scratch of its product
    const int64_t p8 = (p_tokens + 7) / 8 * 8;
    const int64_t pc = p8 < kTokenChunk ? p8 : kTokenChunk;
    size_t hp = hessian_scratch_bytes(n, p8) + kAlign;
    if (h32 > hp) hp = h32;
    const size_t ht = align_up((size_t)n * pc * sizeof(float)) + hp + 4 * kAlign;
    if (ht > h) h = ht;
  }
  // the prepared inputs of a stand-alone T-update stay in front of any other call's scratch
  const size_t keep = (m > 0) ? align_up((size_t)m * n * sizeof(float)) + update_t_scratch_bytes(m, n, nbits) + 4 * kAlign : 0;
  return q > keep + h ? q : keep + h;
}

ganq_status ganq_set_workspace(ganq_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, (dev_ptr != nullptr) == (bytes != 0), "workspace pointer and size disagree");
  GANQ_REQUIRE(ctx, ((uintptr_t)dev_ptr) % kAlign == 0, "workspace must be 256-byte aligned");
  ctx->ws = dev_ptr;
  ctx->ws_bytes = bytes;
  ctx->tprep.valid = false;
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_outlier_split(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m, int64_t n,
                               int64_t ldw, double r, float* W_dense, int64_t ldd, int64_t* row_ptr,
                               int32_t* col_idx, float* values, int64_t capacity, int64_t* nnz_host) {
  return outlier_split_impl(ctx, W, w_dtype, m, n, ldw, r, W_dense, ldd, row_ptr, col_idx, values, capacity,
                            nnz_host, false);
}

ganq_status ganq_outlier_split_noalloc(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                       int64_t n, int64_t ldw, double r, float* W_dense, int64_t ldd,
                                       int64_t* row_ptr, int32_t* col_idx, float* values,
                                       int64_t capacity, int64_t* nnz_host) {
  return outlier_split_impl(ctx, W, w_dtype, m, n, ldw, r, W_dense, ldd, row_ptr, col_idx, values, capacity,
                            nnz_host, true);
}

int64_t ganq_packed_row_bytes(int64_t n, int nbits) {
  if (n <= 0 || n > ((int64_t)1 << 40) || nbits < 1 || nbits > 4) return 0;
  return packed_row_bytes(n, nbits);
}

ganq_status ganq_pack_layer(ganq_ctx* ctx, const uint8_t* Q, int64_t m, int64_t n, int64_t ldq,
                            const float* T, int nbits, uint8_t* packed, int64_t ldp, uint16_t* lut) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, nbits >= 1 && nbits <= 4, "nbits must be 1..4");
  GANQ_REQUIRE(ctx, m > 0 && n > 0, "m and n must be positive");
  GANQ_REQUIRE(ctx, Q != nullptr && ldq >= n, "Q / ldq");
  GANQ_REQUIRE(ctx, T != nullptr && lut != nullptr, "T / lut");
  GANQ_REQUIRE(ctx, packed != nullptr && ((uintptr_t)packed % 16) == 0, "packed must be 16-byte aligned");
  GANQ_REQUIRE(ctx, ldp % 16 == 0 && ldp >= packed_row_bytes(n, nbits), "ldp");
  if (m > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  {
    ProfScope prof(ctx, GANQ_K_PACK);
    GANQ_HIP(ctx, launch_pack_layer(ctx->stream, Q, m, n, ldq, T, nbits, packed, ldp, lut));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_lut_gemv(ganq_ctx* ctx, const uint8_t* packed, int64_t ldp, const uint16_t* lut,
                          int nbits, int64_t m, int64_t n, const void* x, float* y,
                          const int64_t* row_ptr, const int32_t* col_idx, const float* values) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, nbits >= 1 && nbits <= 4, "nbits must be 1..4");
  GANQ_REQUIRE(ctx, m > 0 && n > 0, "m and n must be positive");
  GANQ_REQUIRE(ctx, packed != nullptr && ((uintptr_t)packed % 16) == 0, "packed must be 16-byte aligned");
  GANQ_REQUIRE(ctx, ldp % 16 == 0 && ldp >= packed_row_bytes(n, nbits), "ldp");
  GANQ_REQUIRE(ctx, lut != nullptr && x != nullptr && y != nullptr, "lut / x / y");
  GANQ_REQUIRE(ctx, ((uintptr_t)x % 2) == 0, "x must be 2-byte aligned");
  const bool sparse = row_ptr != nullptr;
  GANQ_REQUIRE(ctx, sparse == (col_idx != nullptr) && sparse == (values != nullptr),
               "row_ptr, col_idx and values go together");
  if (m > (int64_t)kMaxDim * 16) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m must not exceed 1048560");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  {
    ProfScope prof(ctx, GANQ_K_LUT_GEMV);
    GANQ_HIP(ctx, launch_lut_gemv(ctx->stream, packed, ldp, lut, nbits, m, n, (const _Float16*)x, y, row_ptr,
                                  col_idx, values));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_profile_enable(ganq_ctx* ctx, int on) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  if (ctx->device_ready && !ctx->prof_pending.empty()) {
    GANQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
    prof_drain(ctx);
  }
  ctx->prof_on = on != 0;
  for (int k = 0; k < GANQ_K_COUNT; ++k) {
    ctx->prof_ms[k] = 0.0;
    ctx->prof_launches[k] = 0;
  }
  return GANQ_OK;
}

ganq_status ganq_profile_read(ganq_ctx* ctx, double* ms_host, int64_t* launches_host) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, ms_host != nullptr && launches_host != nullptr, "output arrays");
  if (!ctx->prof_pending.empty()) {
    ganq_status st = bind_device(ctx);
    if (st != GANQ_OK) return st;
    GANQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
    prof_drain(ctx);
  }
  for (int k = 0; k < GANQ_K_COUNT; ++k) {
    ms_host[k] = ctx->prof_ms[k];
    launches_host[k] = ctx->prof_launches[k];
  }
  return GANQ_OK;
}

ganq_status ganq_sweep_log(const ganq_ctx* ctx, int32_t* log_host, int capacity, int* sweeps_host) {
  if (ctx == nullptr || sweeps_host == nullptr || capacity < 0) return GANQ_ERR_INVALID_ARG;
  *sweeps_host = ctx->sweep_log_len;
  if (log_host == nullptr) return GANQ_OK;
  for (int k = 0; k < ctx->sweep_log_len && k < capacity; ++k)
    for (int q = 0; q < 3; ++q) log_host[3 * k + q] = ctx->sweep_log[3 * k + q];
  return GANQ_OK;
}

ganq_status ganq_measure_peaks(ganq_ctx* ctx, double* peaks_host) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, peaks_host != nullptr, "peaks_host");
  for (int k = 0; k < 4; ++k) peaks_host[k] = 0.0;
  if (ctx->ws == nullptr || ctx->ws_bytes < ((size_t)2 << 20))
    return fail(ctx, GANQ_ERR_WORKSPACE, "ganq_measure_peaks needs a workspace of at least 2 MiB");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  size_t half = ctx->ws_bytes / 2;
  if (half > ((size_t)1 << 30)) half = (size_t)1 << 30;
  half &= ~(size_t)255;
  hipEvent_t a = nullptr, b = nullptr;
  GANQ_HIP(ctx, hipEventCreate(&a));
  hipError_t e = hipEventCreate(&b);
  if (e != hipSuccess) {
    hipEventDestroy(a);
    return hip_fail(ctx, e, "hipEventCreate");
  }
  for (int which = 0; which < 4 && e == hipSuccess; ++which) {
    double best = 0.0;
    for (int rep = 0; rep < 4 && e == hipSuccess; ++rep) {       // the first launch warms up
      double ops = 0.0;
      float ms = 0.f;
      if ((e = hipEventRecord(a, s)) != hipSuccess) break;
      if ((e = launch_peak_probe(s, which, ctx->ws, half, &ops)) != hipSuccess) break;
      if ((e = hipEventRecord(b, s)) != hipSuccess) break;
      if ((e = hipEventSynchronize(b)) != hipSuccess) break;
      if ((e = hipEventElapsedTime(&ms, a, b)) != hipSuccess) break;
      const double rate = (which < 3) ? ops / (ms * 1e-3) / 1e12 : ops / (ms * 1e-3) / 1e9;
      if (rep > 0 && rate > best) best = rate;
    }
    peaks_host[which] = best;
  }
  hipEventDestroy(a);
  hipEventDestroy(b);
  if (e != hipSuccess) return hip_fail(ctx, e, "peak probe");
  ctx->last_error.clear();
  return GANQ_OK;
}

const char* ganq_status_string(ganq_status s) {
  switch (s) {
    case GANQ_OK: return "ok";
    case GANQ_ERR_INVALID_ARG: return "invalid argument";
    case GANQ_ERR_UNSUPPORTED: return "unsupported";
    case GANQ_ERR_NOT_PD: return "matrix not positive definite";
    case GANQ_ERR_WORKSPACE: return "workspace missing or too small";
    case GANQ_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* ganq_last_error(const ganq_ctx* ctx) {
  return ctx == nullptr ? "" : ctx->last_error.c_str();
}

ganq_status ganq_build_hessian(ganq_ctx* ctx, const void* X, ganq_dtype x_dtype, int64_t n,
                               int64_t p, int64_t ldx, float* H, int64_t ldh, int accumulate) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, dtype_ok(x_dtype), "x_dtype");
  GANQ_REQUIRE(ctx, n > 0 && p >= 0, "n must be positive and p non-negative");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, p == 0 || (X != nullptr && ldx >= p), "X / ldx");
  if (x_dtype == GANQ_F16 && p > 0) {
    if (p % 8 != 0 || ldx % 8 != 0 || ((uintptr_t)X) % 16 != 0)
      return fail(ctx, GANQ_ERR_UNSUPPORTED,
                  "fp16 X needs p % 8 == 0, ldx % 8 == 0 and a 16-byte aligned pointer");
    if (ldx >= ((int64_t)1 << 22))
      return fail(ctx, GANQ_ERR_UNSUPPORTED, "fp16 X needs ldx < 2^22 (32-bit offsets inside a 256-row block)");
  }
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  Arena ar = call_arena(ctx, x_dtype == GANQ_F16 ? hessian_scratch_bytes(n, p > 0 ? p : 1)
                                                 : (size_t)n * n * sizeof(float));
  ProfScope prof(ctx, GANQ_K_HESSIAN);
  if (x_dtype == GANQ_F16) {
    float* part = (float*)ar.take(hessian_scratch_bytes(n, p > 0 ? p : 1));
    if (part == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for H = X X^T");
    GANQ_HIP(ctx, launch_hessian_f16(s, (const _Float16*)X, n, p, ldx, H, ldh, accumulate, part));
  } else {
    float* tmp = (float*)ar.take((size_t)n * n * sizeof(float));
    if (tmp == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for H = X X^T");
    GANQ_HIP(ctx, launch_gemm_f32(s, 1, 1, n, n, p, 1.f, (const float*)X, ldx, (const float*)X, ldx,
                                  0.f, tmp, n));
    GANQ_HIP(ctx, launch_mirror_lower(s, H, n, ldh, tmp, n, accumulate));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_build_hessian_tokens(ganq_ctx* ctx, const void* Xt, ganq_dtype x_dtype, int64_t n,
                                      int64_t p, int64_t ldxt, float* H, int64_t ldh,
                                      int accumulate) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, dtype_ok(x_dtype), "x_dtype");
  GANQ_REQUIRE(ctx, n > 0 && p >= 0, "n must be positive and p non-negative");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, p == 0 || (Xt != nullptr && ldxt >= n), "Xt / ldxt");
  if (p == 0) return ganq_build_hessian(ctx, nullptr, x_dtype, n, 0, 0, H, ldh, accumulate);
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  const int eb = (x_dtype == GANQ_F16) ? 2 : 4;
  if (x_dtype == GANQ_F16 && hessian_tokens_direct_ok(Xt, n, p, ldxt)) {
    // the product reads the token-major array as it is (transposing LDS reads): no copy
    ctx->tprep.valid = false;
    Arena ar(ctx->ws, ctx->ws_bytes);
    float* part = (float*)ar.take(hessian_scratch_bytes(n, p));
    if (part == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for H = Xt^T Xt");
    ProfScope prof(ctx, GANQ_K_HESSIAN);
    GANQ_HIP(ctx, launch_hessian_f16_tokens(s, (const _Float16*)Xt, n, p, ldxt, H, ldh, accumulate, part));
    ctx->last_error.clear();
    return GANQ_OK;
  }
  // Tokens per transposed chunk: what the workspace holds beyond the scratch of the product
  // (at least kTokenChunk, which ganq_workspace_bytes guarantees; a larger workspace means
  // fewer, larger products).
  ctx->tprep.valid = false;          // this call sizes its chunks by the whole workspace
  const int64_t p8 = (p + 7) / 8 * 8;
  const size_t part_bytes = (x_dtype == GANQ_F16) ? hessian_scratch_bytes(n, p8) : (size_t)n * n * sizeof(float);
  int64_t chunk = p8 < kTokenChunk ? p8 : kTokenChunk;
  if (ctx->ws_bytes > part_bytes + 4 * kAlign) {
    const int64_t fit = (int64_t)((ctx->ws_bytes - part_bytes - 4 * kAlign) / ((size_t)n * eb)) / 2048 * 2048;
    if (fit > chunk) chunk = fit < p8 ? fit : p8;
  }
  // the fp16 product addresses a 256-row block of its operand with 32-bit byte offsets: the
  // leading dimension of the transposed chunk (= its token count) must stay below 2^22
  constexpr int64_t kMaxChunkF16 = ((int64_t)1 << 22) - 2048;
  if (x_dtype == GANQ_F16 && chunk > kMaxChunkF16) chunk = kMaxChunkF16;
  Arena ar(ctx->ws, ctx->ws_bytes);
  void* Xn = ar.take((size_t)n * chunk * eb);
  float* part = (float*)ar.take(part_bytes);
  if (Xn == nullptr || part == nullptr)
    return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for H = Xt^T Xt");
  ProfScope prof(ctx, GANQ_K_HESSIAN);
  for (int64_t k0 = 0; k0 < p; k0 += chunk) {
    const int64_t pc = (p - k0 < chunk) ? p - k0 : chunk;
    const int64_t pc8 = (pc + 7) / 8 * 8;                 // zero-padded tokens add nothing to H
    const char* src = (const char*)Xt + (size_t)k0 * ldxt * eb;
    GANQ_HIP(ctx, launch_transpose_tokens(s, src, eb, pc, n, ldxt, Xn, pc8));
    const int acc = (accumulate != 0 || k0 > 0) ? 1 : 0;
    if (x_dtype == GANQ_F16) {
      GANQ_HIP(ctx, launch_hessian_f16(s, (const _Float16*)Xn, n, pc8, pc8, H, ldh, acc, part));
    } else {
      GANQ_HIP(ctx, launch_gemm_f32(s, 1, 1, n, n, pc8, 1.f, (const float*)Xn, pc8, (const float*)Xn, pc8,
                                    0.f, part, n));
      GANQ_HIP(ctx, launch_mirror_lower(s, H, n, ldh, part, n, acc));
    }
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_cholesky(ganq_ctx* ctx, const float* H, int64_t n, int64_t ldh,
                          ganq_precond precond, float lambda, float* L, int64_t ldl,
                          int64_t* info_host) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  if (info_host != nullptr) *info_host = 0;
  GANQ_REQUIRE(ctx, n > 0, "n must be positive");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, L != nullptr && ldl >= n, "L / ldl");
  GANQ_REQUIRE(ctx, (const void*)H != (const void*)L, "L may not alias H");
  GANQ_REQUIRE(ctx, precond >= GANQ_PRECOND_NONE && precond <= GANQ_PRECOND_AUTO, "precond");
  GANQ_REQUIRE(ctx, precond != GANQ_PRECOND_LAMBDA || (lambda > 0.f && std::isfinite(lambda)),
               "lambda must be positive and finite");
  if (n > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "n must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  Arena ar = call_arena(ctx, cholesky_scratch_bytes(n));
  st = run_cholesky(ctx, ar, H, n, ldh, precond, lambda, L, ldl, info_host);
  if (st == GANQ_OK) ctx->last_error.clear();
  return st;
}

ganq_status ganq_init_codebooks(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                int64_t n, int64_t ldw, int nbits, ganq_init init, float* T) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, dtype_ok(w_dtype), "w_dtype");
  GANQ_REQUIRE(ctx, m >= 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, init >= GANQ_INIT_QUANTILE_MID && init <= GANQ_INIT_MINMAX_GRID, "init");
  GANQ_REQUIRE(ctx, m == 0 || (W != nullptr && T != nullptr && ldw >= n), "W / T / ldw");
  if (n > 32768) return fail(ctx, GANQ_ERR_UNSUPPORTED, "init_codebooks supports n <= 32768");
  if (m == 0) return GANQ_OK;
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  {
    ProfScope prof(ctx, GANQ_K_INIT);
    GANQ_HIP(ctx, launch_init_codebooks(ctx->stream, W, w_dtype == GANQ_F16, m, n, ldw, nbits,
                                        (int)init, T));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_update_S(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                          const float* L, int64_t ldl, const float* T, int nbits, uint8_t* Q,
                          int64_t ldq, float* E, int64_t lde) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, m >= 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, L != nullptr && ldl >= n, "L / ldl");
  GANQ_REQUIRE(ctx, m == 0 || (W != nullptr && T != nullptr && Q != nullptr), "W / T / Q");
  GANQ_REQUIRE(ctx, ldw >= n && ldq >= n, "ldw / ldq");
  GANQ_REQUIRE(ctx, E == nullptr || lde >= n, "lde");
  if ((uint64_t)n * (uint64_t)ldl * sizeof(float) >= (1ull << 32))
    return fail(ctx, GANQ_ERR_UNSUPPORTED, "update_S addresses L with 32-bit byte offsets: n * ldl * 4 must stay below 4 GiB");
  if (m == 0) return GANQ_OK;
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  Arena ar = call_arena(ctx, update_s_scratch_bytes(m, n));
  void* scratch = ar.take(update_s_scratch_bytes(m, n));
  if (scratch == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for the S-update");
  {
    ProfScope prof(ctx, GANQ_K_UPDATE_S);
    GANQ_HIP(ctx, launch_update_S(ctx->stream, W, m, n, ldw, L, ldl, T, nbits, Q, ldq, E, lde, scratch));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_update_T_prepare(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                  const float* H, int64_t ldh, int nbits) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  ctx->tprep.valid = false;
  if (W == nullptr && H == nullptr) {          // drop what was prepared
    ctx->last_error.clear();
    return GANQ_OK;
  }
  GANQ_REQUIRE(ctx, m > 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, W != nullptr && ldw >= n, "W / ldw");
  if (m > kMaxDim || n > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m and n must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  Arena ar(ctx->ws, ctx->ws_bytes);
  float* G = (float*)ar.take((size_t)m * n * sizeof(float));
  void* scratch = ar.take(update_t_scratch_bytes(m, n, nbits));
  const size_t keep = ar.off;                   // what stays between calls
  void* gs = ar.take(gemm_split_scratch_bytes(m, n, n));
  if (G == nullptr || scratch == nullptr || gs == nullptr)
    return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for the T-update");
  hipStream_t s = ctx->stream;
  {
    ProfScope prof(ctx, GANQ_K_GEMM_WH);
    GANQ_HIP(ctx, launch_gemm_split(s, m, n, n, W, ldw, H, ldh, G, n, gs, 0));
  }
  {
    ProfScope prof(ctx, GANQ_K_T_PREP);
    GANQ_HIP(ctx, launch_t_prepare(s, H, m, n, ldh, nbits, scratch, 0));
  }
  auto& tp = ctx->tprep;
  tp.W = W; tp.H = H; tp.ldw = ldw; tp.ldh = ldh; tp.m = m; tp.n = n; tp.nbits = nbits;
  tp.ws = ctx->ws; tp.bytes = keep; tp.G = G; tp.t_scratch = scratch;
  tp.valid = true;
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_update_T(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                          const float* H, int64_t ldh, const uint8_t* Q, int64_t ldq, int nbits,
                          ganq_empty empty, float* T, int32_t* empty_count) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, m >= 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, m == 0 || (W != nullptr && T != nullptr && Q != nullptr), "W / T / Q");
  GANQ_REQUIRE(ctx, ldw >= n && ldq >= n, "ldw / ldq");
  GANQ_REQUIRE(ctx, empty == GANQ_EMPTY_ZERO || empty == GANQ_EMPTY_KEEP, "empty");
  if (m == 0) return GANQ_OK;
  if (m > kMaxDim || n > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m and n must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  float* G = nullptr;
  void* scratch = nullptr;
  const auto& tp = ctx->tprep;
  if (tp.valid && tp.ws == ctx->ws && tp.W == (const void*)W && tp.H == (const void*)H && tp.ldw == ldw &&
      tp.ldh == ldh && tp.m == m && tp.n == n && tp.nbits == nbits) {
    // G = W H and the digits of H were left in the workspace by ganq_update_T_prepare
    G = tp.G;
    scratch = tp.t_scratch;
  } else {
    Arena ar = call_arena(ctx, align_up((size_t)m * n * sizeof(float)) + update_t_scratch_bytes(m, n, nbits) +
                                   gemm_split_scratch_bytes(m, n, n) + 4 * kAlign);
    G = (float*)ar.take((size_t)m * n * sizeof(float));
    scratch = ar.take(update_t_scratch_bytes(m, n, nbits));
    void* gs = ar.take(gemm_split_scratch_bytes(m, n, n));
    if (G == nullptr || scratch == nullptr || gs == nullptr)
      return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small for the T-update");
    {
      ProfScope prof(ctx, GANQ_K_GEMM_WH);
      GANQ_HIP(ctx, launch_gemm_split(s, m, n, n, W, ldw, H, ldh, G, n, gs, 0));
    }
    {
      ProfScope prof(ctx, GANQ_K_T_PREP);
      GANQ_HIP(ctx, launch_t_prepare(s, H, m, n, ldh, nbits, scratch, 0));
    }
  }
  {
    ProfScope prof(ctx, GANQ_K_T_PAD);
    GANQ_HIP(ctx, launch_t_pad(s, Q, m, n, ldq, nbits, scratch, 0));
  }
  {
    ProfScope prof(ctx, GANQ_K_T_ACCUM);
    GANQ_HIP(ctx, launch_t_accum(s, m, n, nbits, scratch, 0));
  }
  {
    ProfScope prof(ctx, GANQ_K_T_SOLVE);
    GANQ_HIP(ctx, launch_t_solve(s, G, n, m, n, Q, ldq, nbits, (int)empty, T, empty_count, scratch, -1));
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

ganq_status ganq_layer_loss(ganq_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                            const float* H, int64_t ldh, const float* T, const uint8_t* Q,
                            int64_t ldq, int nbits, double* loss_host, float* row_loss) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  GANQ_REQUIRE(ctx, m >= 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, loss_host != nullptr, "loss_host");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, m == 0 || (W != nullptr && T != nullptr && Q != nullptr), "W / T / Q");
  GANQ_REQUIRE(ctx, ldw >= n && ldq >= n, "ldw / ldq");
  *loss_host = 0.0;
  if (m == 0) return GANQ_OK;
  if (m > kMaxDim || n > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m and n must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  Arena ar = call_arena(ctx, loss_scratch_bytes(m, n) + gemm_split_scratch_bytes(m, n, n) + 4 * kAlign);
  st = run_loss(ctx, ar, W, m, n, ldw, H, ldh, T, Q, ldq, nbits, loss_host, row_loss);
  if (st == GANQ_OK) ctx->last_error.clear();
  return st;
}

ganq_status ganq_quantize_layer(ganq_ctx* ctx, const void* W, ganq_dtype w_dtype, int64_t m,
                                int64_t n, int64_t ldw, const float* H, int64_t ldh,
                                const float* L, int64_t ldl, int nbits, int iters,
                                const ganq_options* opts, float* T, uint8_t* Q, int64_t ldq,
                                double* loss_history_host) {
  if (ctx == nullptr) return GANQ_ERR_INVALID_ARG;
  ganq_options o;
  o.precond = GANQ_PRECOND_NONE;
  o.lambda = 0.f;
  o.init = GANQ_INIT_QUANTILE_MID;
  o.init_codebooks = 0;
  o.empty = GANQ_EMPTY_ZERO;
  o.flags = 0;
  if (opts != nullptr) o = *opts;
  GANQ_REQUIRE(ctx, dtype_ok(w_dtype), "w_dtype");
  GANQ_REQUIRE(ctx, m >= 0 && n > 0, "m, n");
  GANQ_REQUIRE(ctx, nbits_ok(nbits), "nbits must be in [1, 4]");
  GANQ_REQUIRE(ctx, iters >= 0, "iters");
  GANQ_REQUIRE(ctx, H != nullptr && ldh >= n, "H / ldh");
  GANQ_REQUIRE(ctx, L == nullptr || ldl >= n, "ldl");
  GANQ_REQUIRE(ctx, m == 0 || (W != nullptr && T != nullptr && Q != nullptr), "W / T / Q");
  GANQ_REQUIRE(ctx, ldw >= n && ldq >= n, "ldw / ldq");
  GANQ_REQUIRE(ctx, (o.flags & ~GANQ_OPT_FULL_T_UPDATE) == 0, "options.flags has unknown bits");
  GANQ_REQUIRE(ctx, o.precond >= GANQ_PRECOND_NONE && o.precond <= GANQ_PRECOND_AUTO, "options.precond");
  GANQ_REQUIRE(ctx, o.precond != GANQ_PRECOND_LAMBDA || (o.lambda > 0.f && std::isfinite(o.lambda)),
               "options.lambda must be positive and finite");
  GANQ_REQUIRE(ctx, o.init >= GANQ_INIT_QUANTILE_MID && o.init <= GANQ_INIT_MINMAX_GRID, "options.init");
  GANQ_REQUIRE(ctx, o.empty == GANQ_EMPTY_ZERO || o.empty == GANQ_EMPTY_KEEP, "options.empty");
  if (o.init_codebooks && n > 32768)
    return fail(ctx, GANQ_ERR_UNSUPPORTED, "init_codebooks supports n <= 32768");
  if ((uint64_t)n * (uint64_t)(L != nullptr ? ldl : n) * sizeof(float) >= (1ull << 32))
    return fail(ctx, GANQ_ERR_UNSUPPORTED, "the S-update addresses L with 32-bit byte offsets: n * ldl * 4 must stay below 4 GiB");
  if (m == 0) return GANQ_OK;
  if (m > kMaxDim || n > kMaxDim) return fail(ctx, GANQ_ERR_UNSUPPORTED, "m and n must not exceed 65535");
  ganq_status st = bind_device(ctx);
  if (st != GANQ_OK) return st;
  hipStream_t s = ctx->stream;
  ctx->tprep.valid = false;          // the driver lays out the whole workspace itself
  Arena ar(ctx->ws, ctx->ws_bytes);

  // all scratch is carved before the first launch: with the factorisation done here, the work
  // that does not need L (conversion of W, T^0, G = W H, the split of H) runs on a second stream
  // beside it, so none of these buffers may share space with the factorisation's scratch
  float* Wbuf = nullptr;
  if (w_dtype == GANQ_F16) {
    Wbuf = (float*)ar.take((size_t)m * n * sizeof(float));
    if (Wbuf == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small (W)");
  }
  float* Lbuf = nullptr;
  if (L == nullptr) {
    Lbuf = (float*)ar.take((size_t)n * n * sizeof(float));
    if (Lbuf == nullptr) return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small (L)");
  }
  float* G = (float*)ar.take((size_t)m * n * sizeof(float));
  void* s_scratch = ar.take(update_s_scratch_bytes(m, n));
  void* t_scratch = ar.take(update_t_scratch_bytes(m, n, nbits));
  void* gs = ar.take(gemm_split_scratch_bytes(m, n, n));
  if (G == nullptr || s_scratch == nullptr || t_scratch == nullptr || gs == nullptr)
    return fail(ctx, GANQ_ERR_WORKSPACE, "workspace too small (solver scratch)");

  // later sweeps may update S_i H S_i^T from the changed columns instead of summing it again
  const bool incremental = (o.flags & GANQ_OPT_FULL_T_UPDATE) == 0 && iters > 1;
  const size_t prof_first = ctx->prof_pending.size();
  hipStream_t pre = s;               // stream of the work that does not need L
  const bool forked = L == nullptr;
  if (forked) {
    if (ctx->side == nullptr) GANQ_HIP(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
    if (ctx->fork_ev == nullptr) GANQ_HIP(ctx, hipEventCreateWithFlags(&ctx->fork_ev, hipEventDisableTiming));
    if (ctx->join_ev == nullptr) GANQ_HIP(ctx, hipEventCreateWithFlags(&ctx->join_ev, hipEventDisableTiming));
    pre = ctx->side;
    GANQ_HIP(ctx, hipEventRecord(ctx->fork_ev, s));          // inputs produced earlier on the main stream
    GANQ_HIP(ctx, hipStreamWaitEvent(pre, ctx->fork_ev, 0));
  }
  const float* Wf = (const float*)W;
  int64_t ldwf = ldw;
  hipError_t pe = hipSuccess;        // first error on the second stream; checked after the join
  auto pre_work = [&]() -> hipError_t {
    hipError_t e;
    if (w_dtype == GANQ_F16) {
      ProfScope prof(ctx, GANQ_K_INIT, pre);
      if ((e = launch_convert_f16_f32(pre, (const _Float16*)W, m, n, ldw, Wbuf, n)) != hipSuccess) return e;
    }
    if (o.init_codebooks) {
      ProfScope prof(ctx, GANQ_K_INIT, pre);
      if ((e = launch_init_codebooks(pre, Wf, 0, m, n, ldwf, nbits, (int)o.init, T)) != hipSuccess) return e;
    }
    if (iters > 0) {
      {
        ProfScope prof(ctx, GANQ_K_GEMM_WH, pre);
        if ((e = launch_gemm_split(pre, m, n, n, Wf, ldwf, H, ldh, G, n, gs, 0)) != hipSuccess) return e;
      }
      // the integer digits of H are made once per layer
      ProfScope prof(ctx, GANQ_K_T_PREP, pre);
      if ((e = launch_t_prepare(pre, H, m, n, ldh, nbits, t_scratch, incremental ? 1 : 0)) != hipSuccess) return e;
    }
    return hipSuccess;
  };
  if (w_dtype == GANQ_F16) {
    Wf = Wbuf;
    ldwf = n;
  }
  pe = pre_work();
  if (forked) {
    if (pe == hipSuccess) pe = hipEventRecord(ctx->join_ev, pre);
    int64_t info = 0;
    Arena sub((char*)ctx->ws + align_up(ar.off), ctx->ws_bytes - align_up(ar.off));
    st = run_cholesky(ctx, sub, H, n, ldh, o.precond, o.lambda, Lbuf, n, &info);
    if (st != GANQ_OK || pe != hipSuccess) {
      hipStreamSynchronize(pre);     // nothing of this call may still run when it returns
      if (st != GANQ_OK) return st;
    }
    L = Lbuf;
    ldl = n;
  }
  GANQ_HIP(ctx, pe);
  if (forked) GANQ_HIP(ctx, hipStreamWaitEvent(s, ctx->join_ev, 0));

  for (int k = 0; k < iters; ++k) {
    {
      ProfScope prof(ctx, GANQ_K_UPDATE_S);
      GANQ_HIP(ctx, launch_update_S(s, Wf, m, n, ldwf, L, ldl, T, nbits, Q, ldq, nullptr, 0, s_scratch));
    }
    if (loss_history_host != nullptr) {
      Arena sub((char*)ctx->ws + align_up(ar.off), ctx->ws_bytes - align_up(ar.off));
      st = run_loss(ctx, sub, Wf, m, n, ldwf, H, ldh, T, Q, ldq, nbits, &loss_history_host[2 * k], nullptr, gs);
      if (st != GANQ_OK) return st;
    }
    const int cur = k & 1;
    {
      ProfScope prof(ctx, GANQ_K_T_PAD);
      GANQ_HIP(ctx, launch_t_pad(s, Q, m, n, ldq, nbits, t_scratch, cur));
      if (incremental && k > 0) GANQ_HIP(ctx, launch_t_flips(s, m, n, nbits, t_scratch, cur));
    }
    {
      ProfScope prof(ctx, GANQ_K_T_ACCUM, nullptr, k);
      GANQ_HIP(ctx, launch_t_accum(s, m, n, nbits, t_scratch, cur));
    }
    if (incremental && k > 0) {
      ProfScope prof(ctx, GANQ_K_T_DELTA, nullptr, k);
      GANQ_HIP(ctx, launch_t_delta(s, m, n, nbits, t_scratch, cur));
    }
    {
      ProfScope prof(ctx, GANQ_K_T_SOLVE);
      GANQ_HIP(ctx, launch_t_solve(s, G, n, m, n, Q, ldq, nbits, (int)o.empty, T, nullptr, t_scratch, k));
    }
    if (loss_history_host != nullptr) {
      Arena sub((char*)ctx->ws + align_up(ar.off), ctx->ws_bytes - align_up(ar.off));
      st = run_loss(ctx, sub, Wf, m, n, ldwf, H, ldh, T, Q, ldq, nbits, &loss_history_host[2 * k + 1], nullptr, gs);
      if (st != GANQ_OK) return st;
    }
  }
  GANQ_HIP(ctx, hipStreamSynchronize(s));
  ctx->sweep_log_len = 0;
  if (incremental && iters > 0) {
    // which of the two kernels ran in each sweep is known on the device only
    const int cnt = iters < kTLogMax ? iters : kTLogMax;
    GANQ_HIP(ctx, read_t_log(s, m, n, nbits, t_scratch, ctx->sweep_log, cnt));
    ctx->sweep_log_len = cnt;
    // time the other kernel's immediate return under its own class
    for (size_t r = prof_first; r < ctx->prof_pending.size(); ++r) {
      auto& rec = ctx->prof_pending[r];
      if (rec.tag < 0 || rec.tag >= cnt) continue;
      const bool delta = ctx->sweep_log[3 * rec.tag] != 0;
      if ((rec.cls == GANQ_K_T_ACCUM && delta) || (rec.cls == GANQ_K_T_DELTA && !delta)) {
        ctx->prof_launches[rec.cls] -= 1;
        rec.cls = GANQ_K_T_SKIP;
        ctx->prof_launches[GANQ_K_T_SKIP] += 1;
      }
    }
  }
  ctx->last_error.clear();
  return GANQ_OK;
}

}  // extern "C"
