// Error text, back-end selection (MFMA kernels when the shape allows, the
// generic fp32-FMA kernels otherwise) and the C-ABI wrappers of the single
// operations.
#include "common.h"

#include <stdarg.h>
#include <stdio.h>

#include <mutex>
#include <vector>

namespace bm {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

bm_status hip_fail(hipError_t e, const char* what) {
  set_error("HIP error %d (%s) at %s", (int)e, hipGetErrorString(e), what);
  return BM_ERR_HIP;
}

// ---- profiling -----------------------------------------------------------
namespace {
struct ProfRec { int cls; double work; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
}  // namespace

ProfScope::ProfScope(int cls, double work, hipStream_t stream) : slot(-1), st(stream) {
  if (!g_prof_on) return;
  ProfRec r; r.cls = cls; r.work = work;
  if (hipEventCreate(&r.a) != hipSuccess) return;
  if (hipEventCreate(&r.b) != hipSuccess) { hipEventDestroy(r.a); return; }
  hipEventRecord(r.a, st);
  g_prof.push_back(r);
  slot = (int)g_prof.size() - 1;
}

ProfScope::~ProfScope() {
  if (slot >= 0) hipEventRecord(g_prof[slot].b, st);
}

size_t gemm_scratch_bytes(int layout, int M, int N, int K, int dtype) {
  // an upper bound over both back ends (the choice also depends on strides)
  const size_t g = gemm_generic_scratch_bytes(M, N, K);
  const size_t m = dtype == BM_DTYPE_BF16 ? gemm_mfma_scratch_bytes(layout, M, N, K) : 0;
  return g > m ? g : m;
}

bm_status gemm(int layout, int dtype, int M, int N, int K, const void* A, int lda, const void* B,
               int ldb, void* C, int ldc, const GemmEpilogue& epi, void* scratch,
               size_t scratch_bytes, hipStream_t st) {
  if (M <= 0 || N <= 0) return BM_OK;
  ProfScope prof(PROF_GEMM_NT + layout, 2.0 * M * N * K, st);
  if (gemm_mfma_supported(layout, dtype, M, N, K, lda, ldb, ldc, epi))
    return gemm_mfma(layout, M, N, K, A, lda, B, ldb, C, ldc, epi, scratch, scratch_bytes, st);
  return gemm_generic(layout, dtype, M, N, K, A, lda, B, ldb, C, ldc, epi, scratch, scratch_bytes, st);
}

size_t gemm_tn_pair_scratch_bytes(int K, int M0, int N0, int M1, int N1, int dtype) {
  // run separately the two share the buffer; run together each has its own part
  const size_t a = gemm_scratch_bytes(GEMM_TN, M0, N0, K, dtype), b = gemm_scratch_bytes(GEMM_TN, M1, N1, K, dtype);
  const size_t both = dtype == BM_DTYPE_BF16 ? gemm_mfma_tn_pair_scratch_bytes(K, M0, N0, M1, N1) : 0;
  const size_t one = a > b ? a : b;
  return both > one ? both : one;
}

bm_status gemm_tn_pair(int dtype, int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0,
                       void* C0, int ldc0, int M1, int N1, const void* A1, int lda1, const void* B1, int ldb1,
                       void* C1, int ldc1, void* scratch, size_t scratch_bytes, hipStream_t st) {
  if (dtype == BM_DTYPE_BF16 && K > 0 && M0 > 0 && N0 > 0 && M1 > 0 && N1 > 0) {
    if (gemm_mfma_tn_pair(K, M0, N0, A0, lda0, B0, ldb0, C0, ldc0, M1, N1, A1, lda1, B1, ldb1, C1, ldc1, scratch,
                          scratch_bytes, st, nullptr)) {
      bm_status rc;
      ProfScope prof(PROF_GEMM_TN, 2.0 * K * ((double)M0 * N0 + (double)M1 * N1), st);
      gemm_mfma_tn_pair(K, M0, N0, A0, lda0, B0, ldb0, C0, ldc0, M1, N1, A1, lda1, B1, ldb1, C1, ldc1, scratch,
                        scratch_bytes, st, &rc);
      return rc;
    }
  }
  const GemmEpilogue none;
  BM_RETURN_IF(gemm(GEMM_TN, dtype, M0, N0, K, A0, lda0, B0, ldb0, C0, ldc0, none, scratch, scratch_bytes, st));
  return gemm(GEMM_TN, dtype, M1, N1, K, A1, lda1, B1, ldb1, C1, ldc1, none, scratch, scratch_bytes, st);
}

bm_status gemm_grouped(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                       const void* B, int ldb, void* C, int ldc, const GemmGroups& g, hipStream_t st,
                       const GemmEpilogue* epi) {
  if (M <= 0 || N <= 0) return BM_OK;
  const int rows = layout == GEMM_TN ? K : M;
  if (rows % MOE_PAD) { set_error("grouped gemm: %d rows are not a multiple of %d", rows, MOE_PAD); return BM_ERR_INVALID_ARG; }
  if (layout == GEMM_TN ? (!g.group_rows || g.n_groups < 1) : !g.tile_group) {
    set_error("grouped gemm: group tables are NULL");
    return BM_ERR_INVALID_ARG;
  }
  // algorithmic work: the rows that carry tokens, not the padded capacity
  const double rows_used = g.routed_rows > 0 ? (double)g.routed_rows : (double)rows;
  ProfScope prof(PROF_GEMM_NT + layout, layout == GEMM_TN ? 2.0 * M * N * rows_used : 2.0 * rows_used * N * K, st);
  if (gemm_mfma_grouped_supported(layout, dtype, M, N, K, lda, ldb, ldc))
    return gemm_mfma_grouped(layout, M, N, K, A, lda, B, ldb, C, ldc, g, st, epi);
  if (epi) { set_error("grouped gemm: an epilogue needs the MFMA path"); return BM_ERR_UNSUPPORTED; }
  return gemm_generic_grouped(layout, dtype, M, N, K, A, lda, B, ldb, C, ldc, g, st);
}

}  // namespace bm

using namespace bm;

extern "C" const char* bm_last_error(void) { return g_err; }

extern "C" bm_status bm_profile_begin(void) {
  for (auto& r : g_prof) { hipEventDestroy(r.a); hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof_on = true;
  return BM_OK;
}

extern "C" bm_status bm_profile_end(double* ms, double* work, int64_t* launches) {
  g_prof_on = false;
  BM_ARG_CHECK(ms && work && launches, "bm_profile_end: NULL output");
  for (int c = 0; c < PROF_CLASSES; ++c) { ms[c] = 0; work[c] = 0; launches[c] = 0; }
  bm_status rc = BM_OK;
  for (auto& r : g_prof) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
    if (e != hipSuccess) rc = hip_fail(e, "bm_profile_end");
    ms[r.cls] += t; work[r.cls] += r.work; launches[r.cls] += 1;
    hipEventDestroy(r.a); hipEventDestroy(r.b);
  }
  g_prof.clear();
  return rc;
}

static bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

extern "C" size_t bm_gemm_scratch_bytes(int32_t layout, int32_t M, int32_t N, int32_t K,
                                        int32_t dtype) {
  if (layout < 0 || layout > 2 || M <= 0 || N <= 0 || K <= 0) return 0;
  return gemm_scratch_bytes(layout, M, N, K, dtype);
}

extern "C" bm_status bm_gemm(int32_t layout, int32_t dtype, int32_t M, int32_t N, int32_t K,
                             const void* A, int32_t lda, const void* B, int32_t ldb, void* C,
                             int32_t ldc, const void* bias, void* scratch, size_t scratch_bytes,
                             void* hip_stream) {
  BM_ARG_CHECK(layout >= 0 && layout <= 2, "bm_gemm: layout %d", layout);
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "bm_gemm: dtype %d", dtype);
  BM_ARG_CHECK(M > 0 && N > 0 && K > 0, "bm_gemm: sizes must be positive");
  BM_ARG_CHECK(A && B && C && al16(A) && al16(B) && al16(C), "bm_gemm: NULL or misaligned operand");
  BM_ARG_CHECK(!bias || al16(bias), "bm_gemm: misaligned bias");
  BM_ARG_CHECK(layout != GEMM_TN || !bias, "bm_gemm: bias is not defined for layout TN");
  const int a_cols = layout == GEMM_TN ? M : K, b_cols = layout == GEMM_NT ? K : N;
  BM_ARG_CHECK(lda >= a_cols && ldb >= b_cols && ldc >= N, "bm_gemm: leading dimension too small");
  size_t need = gemm_scratch_bytes(layout, M, N, K, dtype);
  if (need > scratch_bytes || (need && !scratch)) {
    set_error("bm_gemm needs %zu scratch bytes, got %zu", need, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  GemmEpilogue e; e.bias = bias;
  return gemm(layout, dtype, M, N, K, A, lda, B, ldb, C, ldc, e, scratch, scratch_bytes,
              (hipStream_t)hip_stream);
}

static bm_status check_attn(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                            const int32_t* cu_dev, const int32_t* cu_host, int32_t S, int32_t T,
                            int32_t max_seqlen, int32_t ld) {
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "attention: dtype %d", dtype);
  BM_ARG_CHECK(mask == 0 || mask == 1, "attention: mask %d", mask);
  BM_ARG_CHECK(Hq > 0 && Hkv > 0 && dh > 0 && Hq % Hkv == 0, "attention: bad head counts %d/%d", Hq, Hkv);
  BM_ARG_CHECK(S >= 1 && T >= 1 && cu_dev && cu_host, "attention: bad S/T/cu_seqlens");
  BM_ARG_CHECK(cu_host[0] == 0 && cu_host[S] == T, "attention: cu_seqlens must span [0, T]");
  for (int s = 0; s < S; ++s) {
    int L = cu_host[s + 1] - cu_host[s];
    BM_ARG_CHECK(L >= 1 && L <= max_seqlen, "attention: sequence %d has length %d (max_seqlen %d)", s, L, max_seqlen);
  }
  BM_ARG_CHECK(ld >= Hq * dh, "attention: row stride %d too small", ld);
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(ld % vec == 0 && dh % vec == 0, "attention: row stride and head_dim must be multiples of %d", vec);
  return BM_OK;
}

extern "C" bm_status bm_attention_forward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv,
                                          int32_t dh, const void* q, const void* k, const void* v,
                                          int32_t ld_qkv, const int32_t* cu_dev,
                                          const int32_t* cu_host, int32_t S, int32_t T,
                                          int32_t max_seqlen, void* o, float* lse, void* hip_stream) {
  BM_RETURN_IF(check_attn(dtype, mask, Hq, Hkv, dh, cu_dev, cu_host, S, T, max_seqlen, ld_qkv));
  BM_ARG_CHECK(q && k && v && o && lse && al16(q) && al16(k) && al16(v) && al16(o),
               "attention: NULL or misaligned tensor");
  AttnArgs a{dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, cu_dev, cu_host, S, T, max_seqlen};
  return attention_forward(a, o, lse, (hipStream_t)hip_stream);
}

extern "C" size_t bm_attention_backward_scratch_bytes(int32_t Hq, int32_t Hkv, int32_t dh, int32_t T) {
  if (Hq <= 0 || Hkv <= 0 || dh <= 0 || T <= 0) return 0;
  return attention_backward_scratch_bytes(Hq, Hkv, dh, T);
}

extern "C" bm_status bm_attention_backward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv,
                                           int32_t dh, const void* q, const void* k, const void* v,
                                           int32_t ld_qkv, const void* o, const void* d_o,
                                           const float* lse, const int32_t* cu_dev,
                                           const int32_t* cu_host, int32_t S, int32_t T,
                                           int32_t max_seqlen, void* dq, void* dk, void* dv,
                                           int32_t ld_dqkv, void* scratch, size_t scratch_bytes,
                                           void* hip_stream) {
  BM_RETURN_IF(check_attn(dtype, mask, Hq, Hkv, dh, cu_dev, cu_host, S, T, max_seqlen, ld_qkv));
  BM_ARG_CHECK(q && k && v && o && d_o && lse && dq && dk && dv, "attention backward: NULL tensor");
  BM_ARG_CHECK(al16(q) && al16(k) && al16(v) && al16(o) && al16(d_o) && al16(dq) && al16(dk) && al16(dv),
               "attention backward: misaligned tensor");
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(ld_dqkv >= Hq * dh && ld_dqkv % vec == 0, "attention backward: bad gradient row stride");
  size_t need = attention_backward_scratch_bytes(Hq, Hkv, dh, T);
  if (need > scratch_bytes || !scratch) {
    set_error("attention backward needs %zu scratch bytes, got %zu", need, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  AttnArgs a{dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, cu_dev, cu_host, S, T, max_seqlen};
  return attention_backward(a, o, d_o, lse, dq, dk, dv, ld_dqkv, scratch, scratch_bytes,
                            (hipStream_t)hip_stream);
}

// ---- attention backward for callers that cannot allocate ----------------------------------
// The workspace of bm_attention_backward (the delta plane and, for grouped-query attention over
// short packs, the fp32 dK/dV partials) lives in device memory that belongs to the code object.
// Each GPU holds its own copy of the array at its own address; the array's name is only a host
// stand-in, so the device address is looked up once per device and kept.
namespace {
constexpr size_t kStaticScratchBytes = BM_ATTENTION_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};

bm_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return bm::hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) {
    bm::set_error("device ordinal %d outside the %d the static workspace table covers", dev, kMaxDevices);
    return BM_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return bm::hip_fail(e, "hipGetSymbolAddress(static attention workspace)");
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return BM_OK;
}
}  // namespace

extern "C" size_t bm_attention_backward_static_capacity(void) { return kStaticScratchBytes; }

extern "C" bm_status bm_attention_backward_static(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv,
                                                  int32_t dh, const void* q, const void* k, const void* v,
                                                  int32_t ld_qkv, const void* o, const void* d_o,
                                                  const float* lse, const int32_t* cu_dev,
                                                  const int32_t* cu_host, int32_t S, int32_t T,
                                                  int32_t max_seqlen, void* dq, void* dk, void* dv,
                                                  int32_t ld_dqkv, void* hip_stream) {
  if (Hq <= 0 || Hkv <= 0 || dh <= 0 || T <= 0) {
    bm::set_error("attention backward (static workspace): non-positive size");
    return BM_ERR_INVALID_ARG;
  }
  const size_t need = bm::attention_backward_scratch_bytes(Hq, Hkv, dh, T);
  if (need > kStaticScratchBytes) {
    bm::set_error("attention backward (static workspace) needs %zu bytes, the built-in workspace holds %zu; "
                  "use bm_attention_backward with a caller workspace", need, kStaticScratchBytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  void* ws = nullptr;
  BM_RETURN_IF(static_scratch(&ws));
  // every byte the kernels read from the workspace is written earlier in the same call
  // (delta plane by the row-sum kernel, partials by the dK/dV kernel), so nothing is cleared
  return bm_attention_backward(dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, o, d_o, lse, cu_dev, cu_host,
                               S, T, max_seqlen, dq, dk, dv, ld_dqkv, ws, kStaticScratchBytes, hip_stream);
}
