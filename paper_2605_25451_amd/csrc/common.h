// Shared declarations of the gfx950 block library: element types, vector
// loads, wavefront reductions, error plumbing and the internal kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/bigmac_block.h"

namespace bm {

typedef __bf16 bf16_t;

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
bm_status hip_fail(hipError_t e, const char* what);

#define BM_CHECK_HIP(expr)                                         \
  do {                                                             \
    hipError_t _e = (expr);                                        \
    if (_e != hipSuccess) return ::bm::hip_fail(_e, #expr);        \
  } while (0)

#define BM_CHECK_LAUNCH(name)                                      \
  do {                                                             \
    hipError_t _e = hipGetLastError();                             \
    if (_e != hipSuccess) return ::bm::hip_fail(_e, name);         \
  } while (0)

#define BM_RETURN_IF(st)                                           \
  do {                                                             \
    bm_status _s = (st);                                           \
    if (_s != BM_OK) return _s;                                    \
  } while (0)

#define BM_ARG_CHECK(cond, ...)                                    \
  do {                                                             \
    if (!(cond)) {                                                 \
      ::bm::set_error(__VA_ARGS__);                                \
      return BM_ERR_INVALID_ARG;                                   \
    }                                                              \
  } while (0)

// ---------------------------------------------------------------- profiling
// Optional per-kernel-class timing with HIP events recorded on the launch
// stream (bm_profile_begin / bm_profile_end).  Off: a scope costs one branch.
enum { PROF_GEMM_NT = 0, PROF_GEMM_NN, PROF_GEMM_TN, PROF_ATTN_FWD, PROF_ATTN_BWD, PROF_NORM,
       PROF_ELEMENTWISE, PROF_CLASSES };
struct ProfScope {
  int slot;
  hipStream_t st;
  ProfScope(int cls, double work, hipStream_t stream);
  ~ProfScope();
};

// ---------------------------------------------------------------- device helpers
constexpr int WAVE = 64;

template <typename T> struct Elt;
template <> struct Elt<float> {
  static constexpr int VEC = 4;   // elements per 16-byte access
  __device__ static inline float to_f(float v) { return v; }
  __device__ static inline float from_f(float v) { return v; }
};
template <> struct Elt<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static inline float to_f(bf16_t v) { return (float)v; }
  __device__ static inline bf16_t from_f(float v) { return (bf16_t)v; }
};

// 16-byte vector of elements with float views.
template <typename T> struct alignas(16) Vec16 {
  T v[Elt<T>::VEC];
};

template <typename T>
__device__ inline void load16(const T* p, float (&out)[Elt<T>::VEC]) {
  Vec16<T> t = *reinterpret_cast<const Vec16<T>*>(p);
#pragma unroll
  for (int i = 0; i < Elt<T>::VEC; ++i) out[i] = Elt<T>::to_f(t.v[i]);
}

template <typename T>
__device__ inline void store16(T* p, const float (&in)[Elt<T>::VEC]) {
  Vec16<T> t;
#pragma unroll
  for (int i = 0; i < Elt<T>::VEC; ++i) t.v[i] = Elt<T>::from_f(in[i]);
  *reinterpret_cast<Vec16<T>*>(p) = t;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
  return v;
}

// ---------------------------------------------------------------- host helpers
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }
inline size_t elt_size(int dtype) { return dtype == BM_DTYPE_BF16 ? 2 : 4; }

// Bump allocator over the caller's workspace; a null base only measures.
struct Arena {
  char* base;
  size_t off = 0;
  explicit Arena(void* b) : base(static_cast<char*>(b)) {}
  template <typename T = void> T* take(size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return base ? reinterpret_cast<T*>(base + o) : nullptr;
  }
};

// ---------------------------------------------------------------- GEMM
enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };

// Epilogue of C = acc (+bias) (+residual); all optional.
struct GemmEpilogue {
  const void* bias = nullptr;       // [N] storage dtype
  const void* residual = nullptr;   // [M, ldc] storage dtype
  int out_fp32 = 0;                 // write C as fp32 regardless of dtype (NT/NN)
  // SwiGLU backward fused into the input-gradient GEMM of the down projection (bf16 MFMA path,
  // NN layout): the product dA[M,N] is not stored; with the saved pre-activations
  // up[M, 2N] = [g | u] the epilogue writes d_up[M, 2N] = [dA u silu'(g) | dA silu(g)] and the
  // activation a[M,N] = silu(g) u (which the weight-gradient GEMM of the down projection reads).
  const void* swiglu_up = nullptr;  // [M, 2N] storage dtype, row stride 2N
  void* swiglu_dup = nullptr;       // [M, 2N]
  void* swiglu_a = nullptr;         // [M, N]
  // SwiGLU forward fused into the up projection (bf16 MFMA path, NT layout, no bias, N a multiple of
  // 256): C[M, N] = [g | u] is written as usual and the epilogue also writes the activation
  // a[M, N/2] = silu(g) u, taken from the ROUNDED g and u (what a separate pass over C would read).
  // A tile gathers its weight rows from both halves, so that g and u of a column meet in one wavefront.
  void* swiglu_fwd_a = nullptr;     // [M, N/2]
};

size_t gemm_scratch_bytes(int layout, int M, int N, int K, int dtype);
bm_status gemm(int layout, int dtype, int M, int N, int K, const void* A, int lda, const void* B,
               int ldb, void* C, int ldc, const GemmEpilogue& epi, void* scratch,
               size_t scratch_bytes, hipStream_t st);

// Grouped GEMM for the mixture-of-experts FFN: the rows of the activation matrices are
// sorted by expert and every expert's segment is padded to MOE_PAD rows.
//   NT / NN: row block t (MOE_PAD rows) of A and C belongs to group tile_group[t] (-1: no
//            group, the block is skipped); the B matrix of group g starts at B + g*b_stride.
//   TN:      group g contracts over rows [group_rows[g], group_rows[g+1]) of A and B and
//            accumulates into the fp32 matrix at C + g*c_stride.
// M (NT/NN) resp. K (TN) is the padded row capacity, a multiple of MOE_PAD.
constexpr int MOE_PAD = 128;
struct GemmGroups {
  const int32_t* tile_group = nullptr;   // dev [rows / MOE_PAD]     (NT, NN)
  const int32_t* group_rows = nullptr;   // dev [n_groups + 1]       (TN)
  int n_groups = 0;
  long b_stride = 0;                     // elements between the B matrices of two groups (NT, NN)
  long c_stride = 0;                     // elements between the C matrices of two groups (TN)
  long routed_rows = 0;                  // rows that carry tokens (profiling: algorithmic flops)
};
// Two weight gradients over the same rows, C_i[M_i,N_i] += A_i[K,M_i]^T B_i[K,N_i] (fp32 C), as one
// launch when that fills the chip better, else one after the other; scratch as for the larger sum
// of both (gemm_pair_scratch_bytes).
size_t gemm_tn_pair_scratch_bytes(int K, int M0, int N0, int M1, int N1, int dtype);
bm_status gemm_tn_pair(int dtype, int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0,
                       void* C0, int ldc0, int M1, int N1, const void* A1, int lda1, const void* B1, int ldb1,
                       void* C1, int ldc1, void* scratch, size_t scratch_bytes, hipStream_t st);
size_t gemm_mfma_tn_pair_scratch_bytes(int K, int M0, int N0, int M1, int N1);
bool gemm_mfma_tn_pair(int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0, void* C0, int ldc0,
                       int M1, int N1, const void* A1, int lda1, const void* B1, int ldb1, void* C1, int ldc1,
                       void* scratch, size_t scratch_bytes, hipStream_t st, bm_status* rc);
// epi (MFMA path only, the caller checks gemm_mfma_grouped_supported): the SwiGLU epilogues of
// GemmEpilogue, forward on NT (N a multiple of 256) and backward on NN (N a multiple of 256)
bm_status gemm_grouped(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                       const void* B, int ldb, void* C, int ldc, const GemmGroups& g, hipStream_t st,
                       const GemmEpilogue* epi = nullptr);
bool gemm_mfma_grouped_supported(int layout, int dtype, int M, int N, int K, int lda, int ldb, int ldc);
bm_status gemm_mfma_grouped(int layout, int M, int N, int K, const void* A, int lda, const void* B,
                            int ldb, void* C, int ldc, const GemmGroups& g, hipStream_t st,
                            const GemmEpilogue* epi = nullptr);
bm_status gemm_generic_grouped(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                               const void* B, int ldb, void* C, int ldc, const GemmGroups& g,
                               hipStream_t st);

// ---------------------------------------------------------------- mixture of experts
// Device tables of one routed batch (all caller memory, see moe.hip for the layout).
struct MoeTables {
  int cap = 0;                 // padded row capacity, moe_row_capacity(T, E, k)
  float* probs = nullptr;      // [T, E] router probabilities
  int32_t* idx = nullptr;      // [T, k] chosen experts, by descending probability
  float* gate = nullptr;       // [T, k] normalised gates
  int32_t* slot = nullptr;     // [T, k] row of each choice in the expert-sorted layout
  int32_t* row_token = nullptr;   // [cap] token of a row, -1 for padding
  float* row_gate = nullptr;      // [cap] gate of a row
  int32_t* tile_group = nullptr;  // [cap / MOE_PAD] expert of a row block, -1 past the end
  int32_t* expert_rows = nullptr; // [E + 1] padded segment offsets
};
int moe_row_capacity(int T, int E, int k);
size_t moe_layout_scratch_bytes(int T, int E);
bm_status moe_check(int E, int k, int d, int dtype);
bm_status moe_route(const float* logits, int T, int E, int k, float* probs, int32_t* idx, float* gate,
                    hipStream_t st);
bm_status moe_layout(const MoeTables& m, int T, int E, int k, void* scratch, hipStream_t st);
bm_status moe_gather(int dtype, const void* src, const MoeTables& m, int use_gate, void* dst, int d, int T,
                     hipStream_t st);
bm_status moe_combine(int dtype, const void* rows, const MoeTables& m, int use_gate, const void* res,
                      void* out, int T, int k, int d, hipStream_t st);
bm_status moe_router_backward(int dtype, const void* dm, const void* y_rows, const MoeTables& m,
                              void* dlogits, int T, int E, int k, int d, hipStream_t st);

// generic (any shape, fp32 FMA) and MFMA (bf16) back ends
size_t gemm_generic_scratch_bytes(int M, int N, int K);
bm_status gemm_generic(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                       const void* B, int ldb, void* C, int ldc, const GemmEpilogue& epi,
                       void* scratch, size_t scratch_bytes, hipStream_t st);
bool gemm_mfma_supported(int layout, int dtype, int M, int N, int K, int lda, int ldb, int ldc,
                         const GemmEpilogue& epi);
size_t gemm_mfma_scratch_bytes(int layout, int M, int N, int K);
bm_status gemm_mfma(int layout, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                    void* C, int ldc, const GemmEpilogue& epi, void* scratch, size_t scratch_bytes,
                    hipStream_t st);

// ---------------------------------------------------------------- attention
struct AttnArgs {
  int dtype, causal, Hq, Hkv, dh;
  const void *q, *k, *v;   // row stride ld_qkv elements
  int ld_qkv;
  const int32_t* cu_dev;
  const int32_t* cu_host;
  int S, T, max_seqlen;
  // Keys/values packed on their own (one chunk of a context-parallel partition of the same S
  // sequences): offsets, rows, row stride and longest segment.  cu_k_dev == nullptr: they share
  // the queries' packing and row stride.  Under a causal mask both packings must be equal (the
  // chunk attends to itself).  ld_dkv: row stride of dk/dv when it differs from dq's.
  const int32_t* cu_k_dev = nullptr;
  const int32_t* cu_k_host = nullptr;
  int Tk = 0, ld_kv = 0, max_klen = 0, ld_dkv = 0;
  const int32_t* kv_cu_dev() const { return cu_k_dev ? cu_k_dev : cu_dev; }
  const int32_t* kv_cu_host() const { return cu_k_dev ? cu_k_host : cu_host; }
  int kv_T() const { return cu_k_dev ? Tk : T; }
  int kv_ld() const { return cu_k_dev ? ld_kv : ld_qkv; }
  int kv_max_len() const { return cu_k_dev ? max_klen : max_seqlen; }
};
bm_status attention_forward(const AttnArgs& a, void* o, float* lse, hipStream_t st);
size_t attention_backward_scratch_bytes(int Hq, int Hkv, int dh, int T);
size_t attention_backward_scratch_bytes(int Hq, int Hkv, int dh, int Tq, int Tk);
bm_status attention_backward(const AttnArgs& a, const void* o, const void* d_o, const float* lse,
                             void* dq, void* dk, void* dv, int ld_dqkv, void* scratch,
                             size_t scratch_bytes, hipStream_t st);

bm_status attention_forward_generic(const AttnArgs& a, void* o, float* lse, hipStream_t st);
bm_status attention_backward_generic(const AttnArgs& a, const void* o, const void* d_o,
                                     const float* lse, void* dq, void* dk, void* dv, int ld_dqkv,
                                     float* delta, hipStream_t st);

// ---------------------------------------------------------------- elementwise / norms
// seq id of every token: tok_seq[t] = s with cu[s] <= t < cu[s+1]
bm_status launch_tok_seq(const int32_t* cu_dev, int S, int T, int32_t* tok_seq, hipStream_t st);

struct NormArgs {
  int dtype, kind;          // BM_NORM_*
  int T, d;
  float eps;
  const void* gamma = nullptr;
  const void* beta = nullptr;
  const float* mod = nullptr;        // adaLN: fp32 [S, ld_mod]
  int ld_mod = 0, shift_off = 0, scale_off = 0;
  const int32_t* tok_seq = nullptr;
};
// h = N(x); stats[2T] = (mean, rstd) written when write_stats
bm_status norm_forward(const NormArgs& a, const void* x, void* h, float* stats, int write_stats,
                       hipStream_t st);
size_t norm_backward_scratch_bytes(int T, int d);
// dx = dres + dN/dx(dh);  dgamma/dbeta fp32 += (LayerNorm/RMSNorm)
// adaLN: dmod[:, shift_off..] = segsum(dh), dmod[:, scale_off..] = segsum(dh * xhat) (overwrite, fp32)
bm_status norm_backward(const NormArgs& a, const void* x, const float* stats, const void* dh,
                        const void* dres, void* dx, void* h_out, float* dgamma, float* dbeta,
                        float* dsum_res, float* dsum_out, float* dmod, const int32_t* cu_dev, int S,
                        void* scratch, hipStream_t st);

// RoPE in place on the first n_heads heads of each row of qkv; sign=+1 fwd, -1 bwd
bm_status rope_inplace(int dtype, void* qkv, int ld, int T, int n_heads, int dh, float base,
                       const int32_t* cu_dev, const int32_t* tok_seq, float sign, hipStream_t st);

bm_status act_forward(int dtype, int act, const void* up, void* a, int T, int F, hipStream_t st);
bm_status act_backward(int dtype, int act, const void* up, const void* da, void* dup, void* a_out,
                       float* bias_grad, void* scratch, int T, int F, hipStream_t st);

// out[n] += sum_t a[t, n]   (fp32 accumulate, deterministic two-stage)
size_t colsum_scratch_bytes(int T, int N);
bm_status colsum_accumulate(int dtype, const void* a, int lda, int T, int N, float* out,
                            void* scratch, hipStream_t st);
// out[s, n] = sum_{t in s} a[t,n] * b[t,n] (fp32, overwrite) and, when gated != nullptr,
// gated[t, n] = a[t, n] * gate[s, n]; rows are N wide; scratch: segment_scratch_bytes()
size_t segment_scratch_bytes();
bm_status segment_gate(int dtype, const void* a, const void* b, const float* gate, int ld_gate, void* gated,
                       const int32_t* cu_dev, int S, int N, float* out, int ld_out, void* scratch,
                       hipStream_t st);
// out[t, n] = (residual ? residual[t,n] : 0) + a[t, n] * gate[tok_seq[t], n]
bm_status gate_mul(int dtype, const void* a, const float* gate, int ld_gate,
                   const int32_t* tok_seq, const void* residual, void* out, int T, int N,
                   hipStream_t st);
// out = silu(in) (storage dtype) ; dsilu: out = g * silu'(in) with g fp32
bm_status silu_forward(int dtype, const void* in, void* out, long n, hipStream_t st);
bm_status silu_backward_f32(int dtype, const void* in, const float* g, void* out, long n,
                            hipStream_t st);
// fp32 -> storage dtype
bm_status cast_from_f32(int dtype, const float* in, void* out, long n, hipStream_t st);
// fp32 [rows, cols] -> storage dtype [cols, ld_out], columns rows..ld_out-1 zero
bm_status cast_transpose_from_f32(int dtype, const float* in, void* out, int rows, int cols, int ld_out,
                                  hipStream_t st);

}  // namespace bm

// ---------------------------------------------------------------- handoff (executor)
namespace bm {
bm_status row_scatter(int dtype, const void* src, const int32_t* rows, void* dst, int n, int width, hipStream_t st);
bm_status row_gather(int dtype, const void* src, const int32_t* rows, void* dst, int n, int width, hipStream_t st);
bm_status fill_zero(void* p, size_t bytes, hipStream_t st);
bm_status add_inplace(int dtype, void* a, const void* b, long n, hipStream_t st);
size_t loss_scratch_bytes();
// grad = (out - target)/n, *loss = 0.5 * mean((out - target)^2)
bm_status mse_loss(int dtype, const void* out, const void* target, void* grad, long n, float* loss, void* scratch, hipStream_t st);
// *loss = <out, g>
bm_status dot_loss(int dtype, const void* out, const void* g, long n, float* loss, void* scratch, hipStream_t st);
}  // namespace bm
