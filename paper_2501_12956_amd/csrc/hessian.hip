// H = X X^T (Algorithm 1; Eq. (9)) for fp16 activations on the gfx950 matrix
// cores: fp16 x fp16 products, fp32 accumulation (v_mfma_f32_32x32x16_f16).
//
// X is n x p row-major, so both operands of the product are k-contiguous.
// Only the 256 x 256 tiles on or below the diagonal are computed (H is symmetric); the
// token axis is split across workgroups so that small n still fills the chip,
// each split writes its partial tile to scratch, and a second kernel sums the
// partials in a fixed order (bit-reproducible, no float atomics) and writes
// both triangles of H.
//
// Operand tiles go from global memory straight into LDS (buffer_load ... lds): no
// registers are held across the MFMA block and no LDS store instructions are issued.  Such
// a load writes 64 x 16 bytes to consecutive LDS addresses, so the LDS tile cannot be
// padded; instead the 16-byte chunks of a row are stored in an XOR-permuted order
// (chunk c of row r at position c ^ (r & 7)), which the lanes apply on the global side
// when they choose what to fetch and on the LDS side when they read MFMA fragments.
#include "ganq_internal.h"

namespace ganq {
namespace {

constexpr int HT = kHessTile;   // 256 x 256 output tile per workgroup
constexpr int HK = 64;          // tokens per LDS stage: one 128-byte line per row
constexpr int HS = 2;           // LDS stages
constexpr int HROWB = HK * 2;   // bytes per LDS row
constexpr int HTILEB = HT * HROWB;
constexpr int HSTAGEB = 2 * HTILEB;          // A rows + B rows
constexpr int HNW = 8;          // wavefronts: 2 x 4, each 128 x 64 of the tile
constexpr int HDPW = (HT / 8) / HNW;         // direct loads per wavefront, operand and stage

constexpr int TROWB = HT * 2;   // token-major stage: bytes per token row (256 features)

typedef _Float16 half4v __attribute__((ext_vector_type(4)));

// Eight consecutive tokens of one feature from a token-major stage: two transpose reads, tokens
// 0..3 at p and 4..7 four token rows further on.
__device__ inline half8 tr_fragment(const unsigned char* p) {
  typedef short short4v __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) short4v lds_short4;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)p);
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)(p + 4 * TROWB));
  return __builtin_shufflevector(__builtin_bit_cast(half4v, lo), __builtin_bit_cast(half4v, hi), 0, 1, 2, 3, 4,
                                 5, 6, 7);
}

// Tiles (r, c), c <= r < nt, of the lower triangle in Z-order (bits of c and r interleaved, c
// lowest): the t-th one, found by descending the quadtree with closed-form counts.
__device__ inline int zorder_box_count(int r0, int c0, int s, int nt) {
  // pairs with r0 <= r < min(r0 + s, nt), c0 <= c < c0 + s, c <= r: row r holds
  // clamp(r - c0 + 1, 0, s) of them
  const int r1 = (r0 + s < nt) ? r0 + s : nt;
  if (r1 <= r0) return 0;
  const int a = (r0 > c0) ? r0 : c0;
  const int b = (r1 < c0 + s - 1) ? r1 : c0 + s - 1;
  int cnt = 0;
  if (b > a) cnt += (b - a) * (a + b - 2 * c0 + 1) / 2;
  const int f = (r0 > c0 + s - 1) ? r0 : c0 + s - 1;
  if (r1 > f) cnt += (r1 - f) * s;
  return cnt;
}

__device__ inline void zorder_tile(int t, int nt, int& bm, int& bn) {
  int s = 1;
  while (s < nt) s <<= 1;
  int r0 = 0, c0 = 0;
  while (s > 1) {
    s >>= 1;
    int cnt = zorder_box_count(r0, c0, s, nt);
    if (t >= cnt) {
      t -= cnt;
      cnt = zorder_box_count(r0, c0 + s, s, nt);
      if (t < cnt) {
        c0 += s;
      } else {
        t -= cnt;
        cnt = zorder_box_count(r0 + s, c0, s, nt);
        r0 += s;
        if (t >= cnt) {
          t -= cnt;
          c0 += s;
        }
      }
    }
  }
  bm = r0;
  bn = c0;
}

// 8 wavefronts (2 per SIMD) in a 2 x 4 grid, each owning 128 x 64 of the tile as 4 x 2 MFMA
// tiles of 32 x 32 (128 accumulator registers).  Two LDS stages of 64 tokens, one barrier
// per stage: after the barrier the loads of the next stage are issued into the buffer that
// every wavefront has just finished reading, then the current stage is multiplied.
//
// TOK: X is the token-major array Xt (p x n, tokens x features, leading dimension ldx) and
// H = Xt^T Xt.  A stage then holds 64 token rows of 256 features per operand (512-byte rows), and
// the MFMA fragments - 8 consecutive tokens of one feature per lane - are gathered by the LDS
// transpose reads of gfx950 (ds_read_b64_tr_b16: within 16 lanes, lane 4a + b receives element b of
// the 8-byte pieces addressed by lanes a, 4 + a, 8 + a, 12 + a).  Lane 4e + a of a group of 16
// addresses token e of a run of four and features 4a .. 4a + 3 of a run of 16, so lane f of the
// group ends up with tokens 0..3 of feature f.  Both operands take the same path, so the order in
// which tokens land in a fragment is the same on both sides of every product.  16-byte chunk c of
// token row t is stored at position c ^ 2 (t & 3): the four token rows a group reads then fall
// into four different 32-byte bank groups.
template <bool TOK>
__global__ __launch_bounds__(64 * HNW) void hessian_f16_kernel(const _Float16* __restrict__ X, int64_t n,
                                                              int64_t p, int64_t ldx, int64_t chunk,
                                                              int nt, int ntiles, int ngroups, int gsz,
                                                              int nsplit, float* __restrict__ partials) {
  // Workgroups are dealt to the 8 XCDs round-robin by their flat index, so the 32 workgroups
  // with consecutive (blockIdx.x >> 3) run side by side on one XCD.  They take one group of at
  // most 32 tiles of one token split, and the groups are runs of the Z-order of the triangle:
  // a group touches few distinct row blocks of X (8 to 12 for 32 tiles), which its workgroups
  // then share through the XCD's L2 instead of each fetching its own pair.
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int item = (q >> 5) * 8 + xcd, w = q & 31;
  const int split = item / ngroups;
  const int t = (item - split * ngroups) * gsz + w;
  if (split >= nsplit || w >= gsz || t >= ntiles) return;
  int bm, bn;
  zorder_tile(t, nt, bm, bn);
  const int64_t kbeg = (int64_t)split * chunk;
  const int64_t kend = (kbeg + chunk < p) ? kbeg + chunk : p;

  extern __shared__ __attribute__((aligned(16))) unsigned char hsm[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)hsm;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 2, wc = wave & 3;
  const int kh = lane >> 5, l32 = lane & 31;
  const int64_t m0 = (int64_t)bm * HT, n0 = (int64_t)bn * HT;

  int4v rsA, rsB;
  uint32_t voff[HDPW], voffB[HDPW];
  int64_t klane = 0;          // !TOK: first token of this lane's chunk within a stage
  int tlane[HDPW];            // TOK: token row of this lane's chunk within a stage
  if constexpr (!TOK) {
    // descriptors over the row blocks of the two operands: rows >= n read as zero
    const int64_t rowsA = (n - m0 < HT) ? n - m0 : HT, rowsB = (n - n0 < HT) ? n - n0 : HT;
    rsA = make_rsrc(X + m0 * ldx, ((rowsA - 1) * ldx + p) * 2);
    rsB = make_rsrc(X + n0 * ldx, ((rowsB - 1) * ldx + p) * 2);
    // One direct load covers 8 rows x 128 bytes: lane -> row (lane / 8) and LDS chunk position
    // (lane % 8), which holds chunk position ^ (row & 7) of the row.
    const int dr = lane >> 3;
    const int dc = (lane & 7) ^ dr;
#pragma unroll
    for (int j = 0; j < HDPW; ++j) {
      voff[j] = (uint32_t)(((int64_t)((wave + HNW * j) * 8 + dr) * ldx + dc * 8) * 2);
      voffB[j] = voff[j];
      tlane[j] = 0;
    }
    klane = dc * 8;
  } else {
    // Descriptors from (first token of this split, first feature of the block) to the end of Xt, at
    // most 2 GiB, which holds every offset a load of this split uses (checked by the host).  What
    // is read is decided per lane, not by the descriptor: chunks of tokens >= kend and of features
    // >= n (n % 8 == 0, so a chunk is wholly inside or outside) get an offset beyond any descriptor
    // and read zero, so no byte outside Xt's p x n elements is touched.
    const int64_t endel = (p - 1) * ldx + n;                        // elements of Xt that exist
    auto span = [&](int64_t base) {
      const int64_t b = (endel - base) * 2;
      return b <= 0 ? (int64_t)0 : (b > 0x80000000ll ? (int64_t)0x80000000ll : b);
    };
    rsA = make_rsrc(X + kbeg * ldx + m0, span(kbeg * ldx + m0));
    rsB = make_rsrc(X + kbeg * ldx + n0, span(kbeg * ldx + n0));
    // One direct load covers 2 token rows x 512 bytes: lane -> token row (lane / 32) and LDS
    // chunk position (lane % 32), which holds chunk position ^ 2 (token & 3) of the row.
#pragma unroll
    for (int j = 0; j < HDPW; ++j) {
      const int tl = 2 * (wave + HNW * j) + (lane >> 5);
      const int cg = (lane & 31) ^ (2 * (tl & 3));
      const uint32_t vo = (uint32_t)(((int64_t)tl * ldx + cg * 8) * 2);
      voff[j] = (m0 + cg * 8 < n) ? vo : 0x80000000u;
      voffB[j] = (n0 + cg * 8 < n) ? vo : 0x80000000u;
      tlane[j] = tl;
    }
  }

  auto issue = [&](int64_t k0, int st) {
    const uint32_t sbase = lds0 + st * HSTAGEB;
    if constexpr (!TOK) {
      const bool ok = k0 + klane < kend;     // p % 8 == 0: a chunk is wholly inside or outside
      const uint32_t soff = (uint32_t)(k0 * 2);
#pragma unroll
      for (int j = 0; j < HDPW; ++j) {
        const uint32_t vo = ok ? voff[j] : 0x80000000u;   // beyond any descriptor: reads zero
        load16_to_lds(rsA, sbase + (wave + HNW * j) * 1024, vo, soff);
        load16_to_lds(rsB, sbase + HTILEB + (wave + HNW * j) * 1024, vo, soff);
      }
    } else {
      const uint32_t soff = (uint32_t)((k0 - kbeg) * ldx * 2);      // below 2^31: checked by the host
#pragma unroll
      for (int j = 0; j < HDPW; ++j) {
        const bool ok = k0 + tlane[j] < kend;
        load16_to_lds(rsA, sbase + (wave + HNW * j) * 1024, ok ? voff[j] : 0x80000000u, soff);
        load16_to_lds(rsB, sbase + HTILEB + (wave + HNW * j) * 1024, ok ? voffB[j] : 0x80000000u, soff);
      }
    }
  };

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int rswz = l32 & 7;
  // TOK: byte offset, inside a stage, of this lane's 8-byte piece for each of the wavefront's
  // fragments: token row 8 (lane / 32) + e, chunk (feature / 8) ^ 2 e, half chunk a & 1
  uint32_t toffA[4], toffB[2];
  {
    const int s16 = lane & 15, e = s16 >> 2, a = s16 & 3, g1 = (lane >> 4) & 1;
    const uint32_t rowb = (uint32_t)((8 * kh + e) * TROWB + 8 * (a & 1));
#pragma unroll
    for (int i = 0; i < 4; ++i)
      toffA[i] = rowb + (uint32_t)(((wr * 16 + i * 4 + 2 * g1 + (a >> 1)) ^ (2 * e)) * 16);
#pragma unroll
    for (int j = 0; j < 2; ++j)
      toffB[j] = rowb + (uint32_t)(((wc * 8 + j * 4 + 2 * g1 + (a >> 1)) ^ (2 * e)) * 16);
  }
  const int nk = (int)((kend - kbeg + HK - 1) / HK);
  if (nk > 0) issue(kbeg, 0);
  int st = 0;
#pragma unroll 1
  for (int k = 0; k < nk; ++k) {
    wait_all_loads();
    __syncthreads();
    if (k + 1 < nk) issue(kbeg + (int64_t)(k + 1) * HK, st ^ 1);
    const unsigned char* As = hsm + st * HSTAGEB;
    const unsigned char* Bs = As + HTILEB;
#pragma unroll
    for (int ks = 0; ks < HK / 16; ++ks) {
      half8 af[4], bfr[2];
      if constexpr (!TOK) {
        const int cpos = ((2 * ks + kh) ^ rswz) * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          af[i] = *reinterpret_cast<const half8*>(As + (wr * 128 + i * 32 + l32) * HROWB + cpos);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          bfr[j] = *reinterpret_cast<const half8*>(Bs + (wc * 64 + j * 32 + l32) * HROWB + cpos);
      } else {
        const unsigned char* Ak = As + ks * (16 * TROWB);
        const unsigned char* Bk = Bs + ks * (16 * TROWB);
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = tr_fragment(Ak + toffA[i]);
#pragma unroll
        for (int j = 0; j < 2; ++j) bfr[j] = tr_fragment(Bk + toffB[j]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    st ^= 1;
  }

  float* out = partials + (int64_t)split * n * n;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t col = n0 + wc * 64 + j * 32 + l32;
      if (col >= n) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wr * 128 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
        if (row < n && col <= row) out[row * n + col] = acc[i][j][v];
      }
    }
}

// H[i][j] = H[j][i] = (accumulate ? H[i][j] : 0) + sum_s src[s][i][j] for i >= j.
__global__ __launch_bounds__(256) void reduce_mirror_kernel(float* __restrict__ H, int64_t n,
                                                            int64_t ldh,
                                                            const float* __restrict__ src,
                                                            int64_t lds, int nsplit,
                                                            int accumulate) {
  const int bi = blockIdx.y, bj = blockIdx.x;
  if (bj > bi) return;
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int64_t i = (int64_t)bi * 32 + r, j = (int64_t)bj * 32 + tx;
    float v = 0.f;
    if (i < n && j < n && j <= i) {
      // four independent running sums keep several loads in flight; the order is fixed
      const float* __restrict__ sp = src + i * lds + j;
      const int64_t ss = lds * n;
      float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
      int s = 0;
      for (; s + 4 <= nsplit; s += 4) {
        v0 += sp[(int64_t)s * ss];
        v1 += sp[(int64_t)(s + 1) * ss];
        v2 += sp[(int64_t)(s + 2) * ss];
        v3 += sp[(int64_t)(s + 3) * ss];
      }
      for (; s < nsplit; ++s) v0 += sp[(int64_t)s * ss];
      v = (v0 + v1) + (v2 + v3);
      if (accumulate) v += H[i * ldh + j];
      H[i * ldh + j] = v;
    }
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    // element (i, j) of the tile goes to H[j][i]; write rows of the transposed tile
    const int64_t jj = (int64_t)bj * 32 + r, ii = (int64_t)bi * 32 + tx;
    if (ii < n && jj < n && jj < ii) H[jj * ldh + ii] = tile[tx][r];
  }
}

// Xn[f][k] = Xt[k][f] for k < pc, 0 for pc <= k < ldn: tokens x features -> features x tokens.
// 64 x 64 tiles through LDS; both sides move 128-byte row segments.
template <typename T>
__global__ __launch_bounds__(256) void transpose_tokens_kernel(const T* __restrict__ Xt, int64_t pc,
                                                               int64_t n, int64_t ldxt,
                                                               T* __restrict__ Xn, int64_t ldn) {
  __shared__ T tile[64][66];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;          // 64 x 4
  const int64_t k0 = (int64_t)blockIdx.x * 64, f0 = (int64_t)blockIdx.y * 64;
#pragma unroll 4
  for (int r = ty; r < 64; r += 4) {
    const int64_t k = k0 + r, f = f0 + tx;
    tile[r][tx] = (k < pc && f < n) ? Xt[k * ldxt + f] : (T)0;
  }
  __syncthreads();
#pragma unroll 4
  for (int r = ty; r < 64; r += 4) {
    const int64_t f = f0 + r, k = k0 + tx;
    if (f < n && k < ldn) Xn[f * ldn + k] = tile[tx][r];
  }
}

}  // namespace

int hessian_split(int64_t n, int64_t p) {
  // about eight workgroups per compute unit, each with at least 2048 tokens
  const int64_t nt = ceil_div(n, HT);
  const int64_t tiles = nt * (nt + 1) / 2;
  int split = 1;
  while (split < kHessMaxSplit && tiles * split < 2048 && p / (split * 2) >= 2048) split *= 2;
  return split;
}

size_t hessian_scratch_bytes(int64_t n, int64_t p) {
  if (p <= 0) return 0;
  return align_up((size_t)hessian_split(n, p) * (size_t)n * (size_t)n * sizeof(float));
}

// Requires p % 8 == 0, ldx % 8 == 0, ldx < 2^22 and a 16-byte aligned X (checked by the caller).
hipError_t launch_hessian_f16(hipStream_t s, const _Float16* X, int64_t n, int64_t p, int64_t ldx,
                              float* H, int64_t ldh, int accumulate, float* partials) {
  if (ldx >= ((int64_t)1 << 22) || (p % 8) != 0 || (ldx % 8) != 0) return hipErrorInvalidValue;
  const int split = hessian_split(n, p);
  int64_t chunk = ceil_div(ceil_div(p, split), HK) * HK;
  const int64_t nt = ceil_div(n, HT);
  const int ntiles = (int)(nt * (nt + 1) / 2);
  const int ngroups = (int)ceil_div(ntiles, 32), gsz = (int)ceil_div(ntiles, ngroups);
  dim3 grid((unsigned)(8 * ceil_div((int64_t)ngroups * split, 8) * 32));
  static std::atomic<uint64_t> lds_set{0};
  {
    const hipError_t ea = ensure_dynamic_lds((const void*)hessian_f16_kernel<false>, HS * HSTAGEB, lds_set);
    if (ea != hipSuccess) return ea;
  }
  hipLaunchKernelGGL(hessian_f16_kernel<false>, grid, dim3(64 * HNW), HS * HSTAGEB, s, X, n, p, ldx, chunk,
                     (int)nt, ntiles, ngroups, gsz, split, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  hipLaunchKernelGGL(reduce_mirror_kernel, g2, dim3(256), 0, s, H, n, ldh, partials, n, split,
                     accumulate);
  return hipGetLastError();
}

// Whether the token-major product can take Xt as it is: 16-byte aligned rows, whole 16-byte chunks
// of features, and a token split whose byte extent fits the 32-bit offsets of the loads.
bool hessian_tokens_direct_ok(const void* Xt, int64_t n, int64_t p, int64_t ldxt) {
  if (p <= 0 || (((uintptr_t)Xt) & 15) != 0 || (ldxt % 8) != 0 || (n % 8) != 0) return false;
  if (ldxt >= ((int64_t)1 << 23)) return false;       // 64 token rows within 31-bit lane offsets
  const int split = hessian_split(n, p);
  const int64_t chunk = ceil_div(ceil_div(p, split), HK) * HK;
  return (chunk + HK) * ldxt * 2 <= ((int64_t)1 << 31);
}

// H (+)= Xt^T Xt straight from the token-major array; requires hessian_tokens_direct_ok.
hipError_t launch_hessian_f16_tokens(hipStream_t s, const _Float16* Xt, int64_t n, int64_t p, int64_t ldxt,
                                     float* H, int64_t ldh, int accumulate, float* partials) {
  if (!hessian_tokens_direct_ok(Xt, n, p, ldxt)) return hipErrorInvalidValue;
  const int split = hessian_split(n, p);
  const int64_t chunk = ceil_div(ceil_div(p, split), HK) * HK;
  const int64_t nt = ceil_div(n, HT);
  const int ntiles = (int)(nt * (nt + 1) / 2);
  const int ngroups = (int)ceil_div(ntiles, 32), gsz = (int)ceil_div(ntiles, ngroups);
  dim3 grid((unsigned)(8 * ceil_div((int64_t)ngroups * split, 8) * 32));
  static std::atomic<uint64_t> lds_set{0};
  {
    const hipError_t ea = ensure_dynamic_lds((const void*)hessian_f16_kernel<true>, HS * HSTAGEB, lds_set);
    if (ea != hipSuccess) return ea;
  }
  hipLaunchKernelGGL(hessian_f16_kernel<true>, grid, dim3(64 * HNW), HS * HSTAGEB, s, Xt, n, p, ldxt, chunk,
                     (int)nt, ntiles, ngroups, gsz, split, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  hipLaunchKernelGGL(reduce_mirror_kernel, g2, dim3(256), 0, s, H, n, ldh, partials, n, split,
                     accumulate);
  return hipGetLastError();
}

hipError_t launch_transpose_tokens(hipStream_t s, const void* Xt, int elem_bytes, int64_t pc, int64_t n,
                                   int64_t ldxt, void* Xn, int64_t ldn) {
  dim3 grid((unsigned)ceil_div(ldn, 64), (unsigned)ceil_div(n, 64));
  if (elem_bytes == 2)
    hipLaunchKernelGGL(transpose_tokens_kernel<_Float16>, grid, dim3(256), 0, s, (const _Float16*)Xt, pc, n,
                       ldxt, (_Float16*)Xn, ldn);
  else
    hipLaunchKernelGGL(transpose_tokens_kernel<float>, grid, dim3(256), 0, s, (const float*)Xt, pc, n, ldxt,
                       (float*)Xn, ldn);
  return hipGetLastError();
}

hipError_t launch_mirror_lower(hipStream_t s, float* H, int64_t n, int64_t ldh, const float* src,
                               int64_t lds, int accumulate) {
  dim3 g2((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  hipLaunchKernelGGL(reduce_mirror_kernel, g2, dim3(256), 0, s, H, n, ldh, src, lds, 1, accumulate);
  return hipGetLastError();
}

}  // namespace ganq
