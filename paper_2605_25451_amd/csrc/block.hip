// bm_block_sizes / bm_block_forward / bm_block_backward: argument checks, the
// layout of the caller's `saved` and `scratch` buffers, and the order in which
// the kernels of one pre-norm transformer block are enqueued.
//
// Saved for backward: norm statistics, post-RoPE qkv, attention output and its
// log-sum-exp, the mid-block residual x1, the MLP pre-activation.  Norm outputs
// and the activation output are not stored: the backward kernels of the norm
// and of the activation write them again next to the gradients they produce.  The adaLN variant also keeps the modulation vectors and
// the two ungated branch outputs (their products with dy give the gate grads).
#include "common.h"

namespace bm {

namespace {

struct Dims {
  int T, S, d, Hq, Hkv, dh, F, QKV, UP, QD;
  size_t es;   // element size
  bool ada;
  int E, k, cap;   // mixture of experts: experts, choices per token, padded row capacity (0 = dense)
};

Dims make_dims(const bm_block_desc& c, int T, int S) {
  Dims m;
  m.T = T; m.S = S; m.d = c.hidden; m.Hq = c.n_q_heads; m.Hkv = c.n_kv_heads; m.dh = c.head_dim;
  m.F = c.mlp_hidden;
  m.QD = m.Hq * m.dh;
  m.QKV = (m.Hq + 2 * m.Hkv) * m.dh;
  m.UP = m.F * (c.act == BM_ACT_SWIGLU ? 2 : 1);
  m.es = elt_size(c.dtype);
  m.ada = c.norm == BM_NORM_ADALN;
  m.E = c.n_experts; m.k = c.top_k;
  m.cap = m.E > 0 ? moe_row_capacity(T, m.E, m.k) : 0;
  return m;
}

struct Saved {
  float *stats1, *stats2, *lse, *mod;
  char *qkv, *o, *x1, *up, *attn, *m;
  MoeTables moe;      // routing tables of the forward pass
  char* moe_y;        // [cap, d] expert outputs in the expert-sorted layout
  size_t bytes;
};

Saved layout_saved(const Dims& m, void* base) {
  Arena a(base);
  Saved s;
  const size_t T = m.T;
  s.stats1 = a.take<float>(2 * T * sizeof(float));
  s.stats2 = a.take<float>(2 * T * sizeof(float));
  s.lse = a.take<float>((size_t)m.Hq * T * sizeof(float));
  s.qkv = a.take<char>(T * m.QKV * m.es);
  s.o = a.take<char>(T * m.QD * m.es);
  s.x1 = a.take<char>(T * m.d * m.es);
  // dense: [T, UP]; experts: [cap, 2F] pre-activations in the expert-sorted layout
  s.up = a.take<char>((m.E > 0 ? (size_t)m.cap : T) * m.UP * m.es);
  s.moe_y = nullptr;
  if (m.E > 0) {
    s.moe.cap = m.cap;
    s.moe.probs = a.take<float>(T * m.E * sizeof(float));
    s.moe.idx = a.take<int32_t>(T * m.k * sizeof(int32_t));
    s.moe.gate = a.take<float>(T * m.k * sizeof(float));
    s.moe.slot = a.take<int32_t>(T * m.k * sizeof(int32_t));
    s.moe.row_token = a.take<int32_t>((size_t)m.cap * sizeof(int32_t));
    s.moe.row_gate = a.take<float>((size_t)m.cap * sizeof(float));
    s.moe.tile_group = a.take<int32_t>((size_t)(m.cap / MOE_PAD) * sizeof(int32_t));
    s.moe.expert_rows = a.take<int32_t>((size_t)(m.E + 1) * sizeof(int32_t));
    s.moe_y = a.take<char>((size_t)m.cap * m.d * m.es);
  }
  s.mod = nullptr; s.attn = nullptr; s.m = nullptr;
  if (m.ada) {
    s.mod = a.take<float>((size_t)m.S * 6 * m.d * sizeof(float));
    s.attn = a.take<char>(T * m.d * m.es);
    s.m = a.take<char>(T * m.d * m.es);
  }
  s.bytes = a.off;
  return s;
}

struct FwdScratch {
  int32_t* tok_seq;
  char *h, *a, *sc;
  float* logits;          // experts: [T, E]
  char *xp, *moe_ws;      // experts: [cap, d] routed inputs; layout scratch
  size_t bytes;
};

FwdScratch layout_fwd(const Dims& m, void* base) {
  Arena a(base);
  FwdScratch s;
  const size_t T = m.T;
  s.tok_seq = a.take<int32_t>(T * sizeof(int32_t));
  s.h = a.take<char>(T * m.d * m.es);
  s.a = a.take<char>((m.E > 0 ? (size_t)m.cap : T) * m.F * m.es);
  s.sc = m.ada ? a.take<char>((size_t)m.S * m.d * m.es) : nullptr;
  s.logits = nullptr; s.xp = nullptr; s.moe_ws = nullptr;
  if (m.E > 0) {
    s.logits = a.take<float>(T * m.E * sizeof(float));
    s.xp = a.take<char>((size_t)m.cap * m.d * m.es);
    s.moe_ws = a.take<char>(moe_layout_scratch_bytes(m.T, m.E));
  }
  s.bytes = a.off;
  return s;
}

struct BwdScratch {
  int32_t* tok_seq;
  char *a, *dup, *da, *h, *dh, *dx1, *dgated, *d_o, *dqkv;
  char *attn_ws, *norm_ws, *colsum_ws, *gemm_ws;
  size_t attn_ws_bytes, gemm_ws_bytes;
  float *dmod, *dsc;
  char *dmod_e, *dmod_t, *sc;
  char *dyp, *xp, *dlogits, *dh2e;   // experts: routed output grads [cap,d], routed inputs [cap,d],
                                     // router logit grads [T,E], expert part of the norm-2 output grad [T,d]
  size_t bytes;
};

size_t max_gemm_tn_scratch(const Dims& m, int dtype) {
  size_t b = 0, v;
  if (m.E > 0) {
    v = gemm_scratch_bytes(GEMM_TN, m.E, m.d, m.T, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_NN, m.T, m.d, m.E, dtype); b = v > b ? v : b;
  } else {
    v = gemm_scratch_bytes(GEMM_TN, m.d, m.F, m.T, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_TN, m.UP, m.d, m.T, dtype); b = v > b ? v : b;
  }
  v = gemm_tn_pair_scratch_bytes(m.T, m.QKV, m.d, m.d, m.QD, dtype); b = v > b ? v : b;
  if (m.ada) {
    v = gemm_scratch_bytes(GEMM_TN, 6 * m.d, m.d, m.S, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_TN, (int)align_up(m.S, 8), m.d, 6 * m.d, dtype); b = v > b ? v : b;
  }
  return b;
}

BwdScratch layout_bwd(const Dims& m, int dtype, void* base) {
  Arena a(base);
  BwdScratch s;
  const size_t T = m.T;
  s.tok_seq = a.take<int32_t>(T * sizeof(int32_t));
  const size_t R = m.E > 0 ? (size_t)m.cap : T;     // rows of the FFN activations
  s.a = a.take<char>(R * m.F * m.es);
  s.dup = a.take<char>(R * m.UP * m.es);
  s.da = a.take<char>(R * m.F * m.es);
  s.h = a.take<char>(T * m.d * m.es);
  s.dh = a.take<char>(T * m.d * m.es);
  s.dx1 = a.take<char>(T * m.d * m.es);
  s.d_o = a.take<char>(T * m.QD * m.es);
  s.dqkv = a.take<char>(T * m.QKV * m.es);
  s.attn_ws_bytes = attention_backward_scratch_bytes(m.Hq, m.Hkv, m.dh, m.T);
  s.attn_ws = a.take<char>(s.attn_ws_bytes);
  s.norm_ws = a.take<char>(norm_backward_scratch_bytes(m.T, m.d));
  int widest = m.UP > m.QKV ? m.UP : m.QKV;
  if (6 * m.d > widest && m.ada) widest = 6 * m.d;
  s.colsum_ws = a.take<char>(colsum_scratch_bytes(m.T, widest));
  s.gemm_ws_bytes = max_gemm_tn_scratch(m, dtype);
  s.gemm_ws = a.take<char>(s.gemm_ws_bytes);
  s.dyp = nullptr; s.xp = nullptr; s.dlogits = nullptr; s.dh2e = nullptr;
  if (m.E > 0) {
    s.dyp = a.take<char>((size_t)m.cap * m.d * m.es);
    s.xp = a.take<char>((size_t)m.cap * m.d * m.es);
    s.dlogits = a.take<char>(T * m.E * m.es);
    s.dh2e = a.take<char>(T * m.d * m.es);
  }
  s.dgated = nullptr; s.dmod = nullptr; s.dsc = nullptr; s.dmod_e = nullptr; s.dmod_t = nullptr; s.sc = nullptr;
  if (m.ada) {
    s.dgated = a.take<char>(T * m.d * m.es);
    s.dmod = a.take<float>((size_t)m.S * 6 * m.d * sizeof(float));
    s.dmod_e = a.take<char>((size_t)m.S * 6 * m.d * m.es);
    s.sc = a.take<char>((size_t)m.S * m.d * m.es);
    const size_t S8 = align_up(m.S, 8);
    s.dmod_t = a.take<char>(S8 * 6 * m.d * m.es);
    s.dsc = a.take<float>(S8 * m.d * sizeof(float));
  }
  s.bytes = a.off;
  return s;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bm_status check_desc(const bm_block_desc* c) {
  BM_ARG_CHECK(c != nullptr, "desc is NULL");
  BM_ARG_CHECK(c->hidden > 0 && c->n_q_heads > 0 && c->n_kv_heads > 0 && c->head_dim > 0 &&
               c->mlp_hidden > 0, "desc: sizes must be positive");
  BM_ARG_CHECK(c->n_q_heads % c->n_kv_heads == 0, "desc: n_q_heads %d not a multiple of n_kv_heads %d",
               c->n_q_heads, c->n_kv_heads);
  BM_ARG_CHECK(c->hidden == c->n_q_heads * c->head_dim, "desc: hidden %d != n_q_heads*head_dim %d",
               c->hidden, c->n_q_heads * c->head_dim);
  BM_ARG_CHECK(c->norm >= 0 && c->norm <= 2, "desc: norm %d", c->norm);
  BM_ARG_CHECK(c->act >= 0 && c->act <= 1, "desc: act %d", c->act);
  BM_ARG_CHECK(c->mask >= 0 && c->mask <= 1, "desc: mask %d", c->mask);
  BM_ARG_CHECK(c->dtype == BM_DTYPE_BF16 || c->dtype == BM_DTYPE_FP32, "desc: dtype %d", c->dtype);
  BM_ARG_CHECK(c->norm_eps >= 0.f, "desc: norm_eps negative");
  BM_ARG_CHECK(!c->rope || c->rope_base > 1.0f, "desc: rope_base must exceed 1");
  const int vec = c->dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (c->hidden % vec || c->mlp_hidden % vec || c->head_dim % vec) {
    set_error("desc: hidden/mlp_hidden/head_dim must be multiples of %d for this dtype", vec);
    return BM_ERR_UNSUPPORTED;
  }
  if (c->rope && (c->head_dim / 2) % vec) {
    set_error("desc: RoPE needs head_dim/2 to be a multiple of %d", vec);
    return BM_ERR_UNSUPPORTED;
  }
  BM_ARG_CHECK(c->n_experts >= 0, "desc: n_experts %d", c->n_experts);
  if (c->n_experts > 0) {
    BM_RETURN_IF(moe_check(c->n_experts, c->top_k, c->hidden, c->dtype));
    if (c->act != BM_ACT_SWIGLU || c->linear_bias || c->norm == BM_NORM_ADALN) {
      set_error("desc: experts need act = SwiGLU, linear_bias = 0 and a norm other than adaLN");
      return BM_ERR_UNSUPPORTED;
    }
  }
  switch (c->head_dim) {
    case 8: case 16: case 32: case 64: case 72: case 128: break;
    default:
      set_error("desc: head_dim %d unsupported (8,16,32,64,72,128)", c->head_dim);
      return BM_ERR_UNSUPPORTED;
  }
  return BM_OK;
}

bm_status check_seqs(const int32_t* cu_dev, const int32_t* cu_host, int S, int T, int max_seqlen) {
  BM_ARG_CHECK(S >= 1 && T >= 1, "S and T must be positive (S=%d, T=%d)", S, T);
  BM_ARG_CHECK(cu_dev && cu_host, "cu_seqlens pointers must not be NULL");
  BM_ARG_CHECK(cu_host[0] == 0, "cu_seqlens[0] = %d, expected 0", cu_host[0]);
  BM_ARG_CHECK(cu_host[S] == T, "cu_seqlens[S] = %d, expected T = %d", cu_host[S], T);
  for (int s = 0; s < S; ++s) {
    int L = cu_host[s + 1] - cu_host[s];
    BM_ARG_CHECK(L >= 1, "sequence %d has length %d (must be >= 1)", s, L);
    BM_ARG_CHECK(L <= max_seqlen, "sequence %d has length %d > max_seqlen %d", s, L, max_seqlen);
  }
  return BM_OK;
}

bm_status check_params(const bm_block_desc& c, const bm_block_params* p, const char* what) {
  BM_ARG_CHECK(p != nullptr, "%s is NULL", what);
  const bool ln = c.norm == BM_NORM_LAYERNORM, rms = c.norm == BM_NORM_RMSNORM, ada = c.norm == BM_NORM_ADALN;
#define NEED(f, cond)                                                                         \
  do {                                                                                        \
    if (cond) {                                                                               \
      BM_ARG_CHECK(p->f != nullptr, "%s.%s is NULL", what, #f);                               \
      BM_ARG_CHECK(aligned16(p->f), "%s.%s is not 16-byte aligned", what, #f);                \
    }                                                                                         \
  } while (0)
  NEED(norm1_g, ln || rms); NEED(norm1_b, ln); NEED(norm2_g, ln || rms); NEED(norm2_b, ln);
  NEED(w_qkv, true); NEED(w_o, true); NEED(w_up, true); NEED(w_down, true);
  NEED(b_qkv, c.linear_bias); NEED(b_o, c.linear_bias); NEED(b_up, c.linear_bias);
  NEED(b_down, c.linear_bias);
  NEED(w_ada, ada); NEED(b_ada, ada);
  NEED(w_router, c.n_experts > 0);
#undef NEED
  return BM_OK;
}

#define NEED_PTR(p)                                                          \
  do {                                                                       \
    BM_ARG_CHECK((p) != nullptr, #p " is NULL");                             \
    BM_ARG_CHECK(aligned16(p), #p " is not 16-byte aligned");                \
  } while (0)

NormArgs norm_args(const bm_block_desc& c, const Dims& m, int which, const bm_block_params* w,
                   const float* mod, const int32_t* tok_seq) {
  NormArgs n;
  n.dtype = c.dtype; n.kind = c.norm; n.T = m.T; n.d = m.d; n.eps = c.norm_eps;
  n.gamma = which == 1 ? w->norm1_g : w->norm2_g;
  n.beta = which == 1 ? w->norm1_b : w->norm2_b;
  n.mod = mod; n.ld_mod = 6 * m.d;
  n.shift_off = which == 1 ? 0 : 3 * m.d;
  n.scale_off = which == 1 ? m.d : 4 * m.d;
  n.tok_seq = tok_seq;
  return n;
}

}  // namespace

}  // namespace bm

using namespace bm;

// No tensor of a call may reach 2^31 elements: the packs the kernels have been exercised on stay
// far below (32768 tokens x 28672 columns), and larger ones are refused rather than trusted.
static bm_status check_extent(const bm_block_desc& c, int T, int S) {
  // the token count alone must leave room for the padded expert capacity of a mixture block
  BM_ARG_CHECK(c.n_experts == 0 || (long)T * c.top_k + (long)c.n_experts * MOE_PAD < (1L << 31),
               "T = %d tokens x %d choices is too large", T, c.top_k);
  const Dims m = make_dims(c, T, S);
  long widest = m.QKV > m.UP ? m.QKV : m.UP;
  if (m.d > widest) widest = m.d;
  const long rows = m.cap > T ? m.cap : T;
  BM_ARG_CHECK(rows * widest < (1L << 31),
               "%ld rows x %ld columns reach 2^31 elements: split the pack", rows, widest);
  return BM_OK;
}

extern "C" bm_status bm_block_sizes(const bm_block_desc* desc, int32_t T, int32_t S,
                                    int32_t max_seqlen, size_t* saved_bytes, size_t* scratch_bytes) {
  BM_RETURN_IF(check_desc(desc));
  BM_ARG_CHECK(T >= 1 && S >= 1 && S <= T && max_seqlen >= 1 && max_seqlen <= T,
               "bm_block_sizes: bad T=%d S=%d max_seqlen=%d", T, S, max_seqlen);
  BM_ARG_CHECK(saved_bytes && scratch_bytes, "bm_block_sizes: output pointers are NULL");
  BM_RETURN_IF(check_extent(*desc, T, S));
  Dims m = make_dims(*desc, T, S);
  *saved_bytes = layout_saved(m, nullptr).bytes;
  size_t f = layout_fwd(m, nullptr).bytes, b = layout_bwd(m, desc->dtype, nullptr).bytes;
  *scratch_bytes = f > b ? f : b;
  return BM_OK;
}

extern "C" bm_status bm_block_moe_routing(const bm_block_desc* desc, int32_t T, int32_t S,
                                          const void* saved, const int32_t** expert_out,
                                          const float** gate_out) {
  BM_RETURN_IF(check_desc(desc));
  BM_ARG_CHECK(desc->n_experts > 0, "bm_block_moe_routing: the block has no experts");
  BM_ARG_CHECK(T >= 1 && S >= 1 && S <= T, "bm_block_moe_routing: bad T=%d S=%d", T, S);
  BM_ARG_CHECK(saved && expert_out && gate_out, "bm_block_moe_routing: NULL pointer");
  BM_RETURN_IF(check_extent(*desc, T, S));
  Saved sv = layout_saved(make_dims(*desc, T, S), const_cast<void*>(saved));
  *expert_out = sv.moe.idx;
  *gate_out = sv.moe.gate;
  return BM_OK;
}

extern "C" bm_status bm_block_forward(const bm_block_desc* desc, const bm_block_params* w,
                                      const void* x, const int32_t* cu_dev, const int32_t* cu_host,
                                      int32_t S, int32_t T, int32_t max_seqlen, const void* cond,
                                      void* y, void* saved, void* scratch, size_t scratch_bytes,
                                      void* hip_stream) {
  BM_RETURN_IF(check_desc(desc));
  const bm_block_desc& c = *desc;
  BM_RETURN_IF(check_seqs(cu_dev, cu_host, S, T, max_seqlen));
  BM_RETURN_IF(check_extent(c, T, S));
  BM_RETURN_IF(check_params(c, w, "w"));
  NEED_PTR(x); NEED_PTR(y); NEED_PTR(saved); NEED_PTR(scratch);
  BM_ARG_CHECK(x != y, "y must not alias x");
  Dims m = make_dims(c, T, S);
  if (m.ada) NEED_PTR(cond);
  FwdScratch ws = layout_fwd(m, scratch);
  if (ws.bytes > scratch_bytes) {
    set_error("forward needs %zu scratch bytes, got %zu", ws.bytes, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  Saved sv = layout_saved(m, saved);
  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c.dtype;

  // token -> sequence map: read by the rotary embedding and by the per-sequence modulation only
  if (c.rope || m.ada) BM_RETURN_IF(launch_tok_seq(cu_dev, S, T, ws.tok_seq, st));
  if (m.ada) {
    BM_RETURN_IF(silu_forward(dt, cond, ws.sc, (long)S * m.d, st));
    GemmEpilogue e; e.bias = w->b_ada; e.out_fp32 = 1;
    BM_RETURN_IF(gemm(GEMM_NT, dt, S, 6 * m.d, m.d, ws.sc, m.d, w->w_ada, m.d, sv.mod, 6 * m.d, e,
                      nullptr, 0, st));
  }
  // attention half
  { ProfScope _p(PROF_NORM, 2.0 * T * m.d * (double)m.es, st); BM_RETURN_IF(norm_forward(norm_args(c, m, 1, w, sv.mod, ws.tok_seq), x, ws.h, sv.stats1, 1, st)); }
  {
    GemmEpilogue e; e.bias = c.linear_bias ? w->b_qkv : nullptr;
    BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.QKV, m.d, ws.h, m.d, w->w_qkv, m.d, sv.qkv, m.QKV, e,
                      nullptr, 0, st));
  }
  if (c.rope)
    { ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * (m.Hq + m.Hkv) * m.dh * (double)m.es, st); BM_RETURN_IF(rope_inplace(dt, sv.qkv, m.QKV, T, m.Hq + m.Hkv, m.dh, c.rope_base, cu_dev,
                              ws.tok_seq, 1.0f, st)); }
  AttnArgs at;
  at.dtype = dt; at.causal = c.mask == BM_MASK_CAUSAL; at.Hq = m.Hq; at.Hkv = m.Hkv; at.dh = m.dh;
  at.q = sv.qkv; at.k = sv.qkv + (size_t)m.QD * m.es; at.v = sv.qkv + (size_t)(m.QD + m.Hkv * m.dh) * m.es;
  at.ld_qkv = m.QKV; at.cu_dev = cu_dev; at.cu_host = cu_host; at.S = S; at.T = T;
  at.max_seqlen = max_seqlen;
  BM_RETURN_IF(attention_forward(at, sv.o, sv.lse, st));
  {
    GemmEpilogue e; e.bias = c.linear_bias ? w->b_o : nullptr;
    if (m.ada) {
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.d, m.QD, sv.o, m.QD, w->w_o, m.QD, sv.attn, m.d, e,
                        nullptr, 0, st));
      { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(gate_mul(dt, sv.attn, sv.mod + 2 * m.d, 6 * m.d, ws.tok_seq, x, sv.x1, T, m.d, st)); }
    } else {
      e.residual = x;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.d, m.QD, sv.o, m.QD, w->w_o, m.QD, sv.x1, m.d, e,
                        nullptr, 0, st));
    }
  }
  // MLP half
  { ProfScope _p(PROF_NORM, 2.0 * T * m.d * (double)m.es, st); BM_RETURN_IF(norm_forward(norm_args(c, m, 2, w, sv.mod, ws.tok_seq), sv.x1, ws.h, sv.stats2, 1, st)); }
  if (m.E > 0) {
    // mixture of experts: route, sort the routed rows by expert, run the expert FFNs as
    // grouped GEMMs over the sorted rows, and sum each token's k gated outputs
    {
      GemmEpilogue e; e.out_fp32 = 1;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.E, m.d, ws.h, m.d, w->w_router, m.d, ws.logits, m.E, e,
                        nullptr, 0, st));
    }
    GemmGroups g;
    g.tile_group = sv.moe.tile_group; g.routed_rows = (long)T * m.k;
    {
      ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(moe_route(ws.logits, T, m.E, m.k, sv.moe.probs, sv.moe.idx, sv.moe.gate, st));
      BM_RETURN_IF(moe_layout(sv.moe, T, m.E, m.k, ws.moe_ws, st));
      BM_RETURN_IF(moe_gather(dt, ws.h, sv.moe, 0, ws.xp, m.d, T, st));
    }
    g.b_stride = (long)m.UP * m.d;
    if (c.act == BM_ACT_SWIGLU && m.UP % 256 == 0 &&
        gemm_mfma_grouped_supported(GEMM_NT, dt, m.cap, m.UP, m.d, m.d, m.d, m.UP)) {
      // the activation rides in the epilogue of the experts' up projections
      GemmEpilogue e; e.swiglu_fwd_a = ws.a;
      BM_RETURN_IF(gemm_grouped(GEMM_NT, dt, m.cap, m.UP, m.d, ws.xp, m.d, w->w_up, m.d, sv.up, m.UP, g, st, &e));
    } else {
      BM_RETURN_IF(gemm_grouped(GEMM_NT, dt, m.cap, m.UP, m.d, ws.xp, m.d, w->w_up, m.d, sv.up, m.UP, g, st));
      { ProfScope _p(PROF_ELEMENTWISE, (double)m.cap * (m.UP + m.F) * (double)m.es, st); BM_RETURN_IF(act_forward(dt, c.act, sv.up, ws.a, m.cap, m.F, st)); }
    }
    g.b_stride = (long)m.d * m.F;
    BM_RETURN_IF(gemm_grouped(GEMM_NT, dt, m.cap, m.d, m.F, ws.a, m.F, w->w_down, m.F, sv.moe_y, m.d, g, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(moe_combine(dt, sv.moe_y, sv.moe, 1, sv.x1, y, T, m.k, m.d, st)); }
    return BM_OK;
  }
  {
    GemmEpilogue e; e.bias = c.linear_bias ? w->b_up : nullptr;
    if (dt == BM_DTYPE_BF16 && c.act == BM_ACT_SWIGLU && !c.linear_bias && m.UP % 256 == 0 &&
        gemm_mfma_supported(GEMM_NT, dt, T, m.UP, m.d, m.d, m.d, m.UP, e)) {
      // the activation rides in the epilogue of the up projection: the pre-activations are not read again
      e.swiglu_fwd_a = ws.a;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.UP, m.d, ws.h, m.d, w->w_up, m.d, sv.up, m.UP, e, nullptr, 0, st));
    } else {
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.UP, m.d, ws.h, m.d, w->w_up, m.d, sv.up, m.UP, e,
                        nullptr, 0, st));
      { ProfScope _p(PROF_ELEMENTWISE, (double)T * (m.UP + m.F) * (double)m.es, st); BM_RETURN_IF(act_forward(dt, c.act, sv.up, ws.a, T, m.F, st)); }
    }
  }
  {
    GemmEpilogue e; e.bias = c.linear_bias ? w->b_down : nullptr;
    if (m.ada) {
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.d, m.F, ws.a, m.F, w->w_down, m.F, sv.m, m.d, e,
                        nullptr, 0, st));
      { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(gate_mul(dt, sv.m, sv.mod + 5 * m.d, 6 * m.d, ws.tok_seq, sv.x1, y, T, m.d, st)); }
    } else {
      e.residual = sv.x1;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.d, m.F, ws.a, m.F, w->w_down, m.F, y, m.d, e,
                        nullptr, 0, st));
    }
  }
  return BM_OK;
}

extern "C" bm_status bm_block_backward(const bm_block_desc* desc, const bm_block_params* w,
                                       const void* x, const void* dy, const int32_t* cu_dev,
                                       const int32_t* cu_host, int32_t S, int32_t T,
                                       int32_t max_seqlen, const void* cond, const void* saved,
                                       void* dx, const bm_block_params* grads, void* dcond,
                                       void* scratch, size_t scratch_bytes, void* hip_stream) {
  BM_RETURN_IF(check_desc(desc));
  const bm_block_desc& c = *desc;
  BM_RETURN_IF(check_seqs(cu_dev, cu_host, S, T, max_seqlen));
  BM_RETURN_IF(check_extent(c, T, S));
  BM_RETURN_IF(check_params(c, w, "w"));
  BM_RETURN_IF(check_params(c, grads, "grads"));
  NEED_PTR(x); NEED_PTR(dy); NEED_PTR(dx); NEED_PTR(saved); NEED_PTR(scratch);
  BM_ARG_CHECK(dx != dy && dx != x, "dx must not alias dy or x");
  Dims m = make_dims(c, T, S);
  if (m.ada) { NEED_PTR(cond); NEED_PTR(dcond); }
  BwdScratch ws = layout_bwd(m, c.dtype, scratch);
  if (ws.bytes > scratch_bytes) {
    set_error("backward needs %zu scratch bytes, got %zu", ws.bytes, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  Saved sv = layout_saved(m, const_cast<void*>(saved));
  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c.dtype;
  const GemmEpilogue none;
  const int d = m.d;

  // token -> sequence map: read by the rotary embedding and by the per-sequence modulation only
  if (c.rope || m.ada) BM_RETURN_IF(launch_tok_seq(cu_dev, S, T, ws.tok_seq, st));

  // ---- y = x1 + [g2 *] m,  m = a W_down^T + b_down
  const void* dm = dy;
  if (m.ada) {
    // gate gradient (per-sequence sum of dy * m) and the gated upstream gradient in one pass over dy
    { ProfScope _p(PROF_ELEMENTWISE, 3.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(segment_gate(dt, dy, sv.m, sv.mod + 5 * d, 6 * d, ws.dgated, cu_dev, S, d, ws.dmod + 5 * d, 6 * d,
                                ws.norm_ws, st)); }
    dm = ws.dgated;
  }
  const bool fused_sums = c.linear_bias && !m.ada;
  if (m.E > 0) {
    // ---- mixture of experts (dm = dy: no gate sits on this branch)
    GemmGroups g;
    g.tile_group = sv.moe.tile_group; g.group_rows = sv.moe.expert_rows; g.n_groups = m.E;
    g.routed_rows = (long)T * m.k;
    {
      ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(moe_gather(dt, dm, sv.moe, 1, ws.dyp, d, T, st));            // gate * dy of the row's token
      BM_RETURN_IF(moe_router_backward(dt, dm, sv.moe_y, sv.moe, ws.dlogits, T, m.E, m.k, d, st));
    }
    g.b_stride = (long)d * m.F;
    if (c.act == BM_ACT_SWIGLU && m.F % 256 == 0 &&
        gemm_mfma_grouped_supported(GEMM_NN, dt, m.cap, m.F, d, d, m.F, m.F)) {
      // SwiGLU backward in the epilogue of the experts' input-gradient GEMM: dA never goes to memory
      GemmEpilogue e; e.swiglu_up = sv.up; e.swiglu_dup = ws.dup; e.swiglu_a = ws.a;
      BM_RETURN_IF(gemm_grouped(GEMM_NN, dt, m.cap, m.F, d, ws.dyp, d, w->w_down, m.F, ws.da, m.F, g, st, &e));
    } else {
      BM_RETURN_IF(gemm_grouped(GEMM_NN, dt, m.cap, m.F, d, ws.dyp, d, w->w_down, m.F, ws.da, m.F, g, st));
      { ProfScope _p(PROF_ELEMENTWISE, (double)m.cap * (2.0 * m.UP + 2.0 * m.F) * (double)m.es, st);
        BM_RETURN_IF(act_backward(dt, c.act, sv.up, ws.da, ws.dup, ws.a, nullptr, ws.colsum_ws, m.cap, m.F, st)); }
    }
    g.c_stride = (long)d * m.F;
    BM_RETURN_IF(gemm_grouped(GEMM_TN, dt, d, m.F, m.cap, ws.dyp, d, ws.a, m.F, grads->w_down, m.F, g, st));
    g.b_stride = (long)m.UP * d;
    char* dxp = ws.dyp;                                  // the routed output gradient is spent
    BM_RETURN_IF(gemm_grouped(GEMM_NN, dt, m.cap, d, m.UP, ws.dup, m.UP, w->w_up, d, dxp, d, g, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(moe_combine(dt, dxp, sv.moe, 0, nullptr, ws.dh2e, T, m.k, d, st)); }
    {
      GemmEpilogue e; e.residual = ws.dh2e;              // + the router's path
      BM_RETURN_IF(gemm(GEMM_NN, dt, T, d, m.E, ws.dlogits, m.E, w->w_router, d, ws.dh, d, e, ws.gemm_ws,
                        ws.gemm_ws_bytes, st));
    }
    NormArgs n2 = norm_args(c, m, 2, w, sv.mod, ws.tok_seq);
    { ProfScope _p(PROF_NORM, 5.0 * T * m.d * (double)m.es, st);
      BM_RETURN_IF(norm_backward(n2, sv.x1, sv.stats2, ws.dh, dy, ws.dx1, ws.h, (float*)grads->norm2_g,
                                 (float*)grads->norm2_b, nullptr, nullptr, ws.dmod, cu_dev, S, ws.norm_ws, st)); }
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(moe_gather(dt, ws.h, sv.moe, 0, ws.xp, d, T, st)); }
    g.c_stride = (long)m.UP * d;
    BM_RETURN_IF(gemm_grouped(GEMM_TN, dt, m.UP, d, m.cap, ws.dup, m.UP, ws.xp, d, grads->w_up, d, g, st));
    BM_RETURN_IF(gemm(GEMM_TN, dt, m.E, d, T, ws.dlogits, m.E, ws.h, d, grads->w_router, d, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
  } else {
  // input gradient first: the activation backward then also rewrites the activation
  // output that the weight-gradient GEMM of the down projection reads
  GemmEpilogue down_in;
  if (dt == BM_DTYPE_BF16 && c.act == BM_ACT_SWIGLU && !c.linear_bias &&
      gemm_mfma_supported(GEMM_NN, dt, T, m.F, d, d, m.F, m.F, down_in)) {
    // SwiGLU backward rides in the epilogue of this GEMM: dA never goes to memory
    down_in.swiglu_up = sv.up; down_in.swiglu_dup = ws.dup; down_in.swiglu_a = ws.a;
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, m.F, d, dm, d, w->w_down, m.F, ws.da, m.F, down_in, nullptr, 0, st));
  } else {
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, m.F, d, dm, d, w->w_down, m.F, ws.da, m.F, none, nullptr, 0, st));
    { ProfScope _p(PROF_ELEMENTWISE, (double)T * (2.0 * m.UP + 2.0 * m.F) * (double)m.es, st);
      BM_RETURN_IF(act_backward(dt, c.act, sv.up, ws.da, ws.dup, ws.a,
                                c.linear_bias ? (float*)grads->b_up : nullptr, ws.colsum_ws, T, m.F, st)); }
  }
  BM_RETURN_IF(gemm(GEMM_TN, dt, d, m.F, T, dm, d, ws.a, m.F, grads->w_down, m.F, none, ws.gemm_ws,
                    ws.gemm_ws_bytes, st));
  // bias gradients of the down and output projections are column sums of the two
  // gradients the norm backward below touches anyway (not so when a gate sits between)
  if (c.linear_bias && !fused_sums)
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(colsum_accumulate(dt, dm, d, T, d, (float*)grads->b_down, ws.colsum_ws, st)); }

  // ---- up = h2 W_up^T + b_up,  h2 = N2(x1)
  NormArgs n2 = norm_args(c, m, 2, w, sv.mod, ws.tok_seq);
  BM_RETURN_IF(gemm(GEMM_NN, dt, T, d, m.UP, ws.dup, m.UP, w->w_up, d, ws.dh, d, none, nullptr, 0, st));
  { ProfScope _p(PROF_NORM, 5.0 * T * m.d * (double)m.es, st);
    BM_RETURN_IF(norm_backward(n2, sv.x1, sv.stats2, ws.dh, dy, ws.dx1, ws.h, (float*)grads->norm2_g,
                               (float*)grads->norm2_b, fused_sums ? (float*)grads->b_down : nullptr,
                               fused_sums ? (float*)grads->b_o : nullptr, ws.dmod, cu_dev, S,
                               ws.norm_ws, st)); }
  BM_RETURN_IF(gemm(GEMM_TN, dt, m.UP, d, T, ws.dup, m.UP, ws.h, d, grads->w_up, d, none, ws.gemm_ws,
                    ws.gemm_ws_bytes, st));

  }

  // ---- x1 = x + [g1 *] attn,  attn = o W_o^T + b_o
  const void* dattn = ws.dx1;
  if (m.ada) {
    { ProfScope _p(PROF_ELEMENTWISE, 3.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(segment_gate(dt, ws.dx1, sv.attn, sv.mod + 2 * d, 6 * d, ws.dgated, cu_dev, S, d, ws.dmod + 2 * d,
                                6 * d, ws.norm_ws, st)); }
    dattn = ws.dgated;
  }
  // (the weight gradient of the output projection is small: it shares a launch with the one of
  // the QKV projection at the end; dattn and the saved o stay untouched until then)
  if (c.linear_bias && !fused_sums)
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(colsum_accumulate(dt, dattn, d, T, d, (float*)grads->b_o, ws.colsum_ws, st)); }
  BM_RETURN_IF(gemm(GEMM_NN, dt, T, m.QD, d, dattn, d, w->w_o, m.QD, ws.d_o, m.QD, none, nullptr, 0, st));

  // ---- attention
  AttnArgs at;
  at.dtype = dt; at.causal = c.mask == BM_MASK_CAUSAL; at.Hq = m.Hq; at.Hkv = m.Hkv; at.dh = m.dh;
  at.q = sv.qkv; at.k = sv.qkv + (size_t)m.QD * m.es; at.v = sv.qkv + (size_t)(m.QD + m.Hkv * m.dh) * m.es;
  at.ld_qkv = m.QKV; at.cu_dev = cu_dev; at.cu_host = cu_host; at.S = S; at.T = T;
  at.max_seqlen = max_seqlen;
  char* dq = ws.dqkv;
  char* dk = ws.dqkv + (size_t)m.QD * m.es;
  char* dv = ws.dqkv + (size_t)(m.QD + m.Hkv * m.dh) * m.es;
  BM_RETURN_IF(attention_backward(at, sv.o, ws.d_o, sv.lse, dq, dk, dv, m.QKV, ws.attn_ws,
                                  ws.attn_ws_bytes, st));
  if (c.rope)
    { ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * (m.Hq + m.Hkv) * m.dh * (double)m.es, st); BM_RETURN_IF(rope_inplace(dt, ws.dqkv, m.QKV, T, m.Hq + m.Hkv, m.dh, c.rope_base, cu_dev,
                              ws.tok_seq, -1.0f, st)); }

  // ---- qkv = h W_qkv^T + b_qkv,  h = N1(x)
  NormArgs n1 = norm_args(c, m, 1, w, sv.mod, ws.tok_seq);
  if (c.linear_bias)
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(colsum_accumulate(dt, ws.dqkv, m.QKV, T, m.QKV, (float*)grads->b_qkv, ws.colsum_ws, st)); }
  BM_RETURN_IF(gemm(GEMM_NN, dt, T, d, m.QKV, ws.dqkv, m.QKV, w->w_qkv, d, ws.dh, d, none, nullptr, 0, st));
  { ProfScope _p(PROF_NORM, 5.0 * T * m.d * (double)m.es, st);
    BM_RETURN_IF(norm_backward(n1, x, sv.stats1, ws.dh, ws.dx1, dx, ws.h, (float*)grads->norm1_g,
                               (float*)grads->norm1_b, nullptr, nullptr, ws.dmod, cu_dev, S,
                               ws.norm_ws, st)); }
  BM_RETURN_IF(gemm_tn_pair(dt, T, m.QKV, d, ws.dqkv, m.QKV, ws.h, d, grads->w_qkv, d,
                            d, m.QD, dattn, d, sv.o, m.QD, grads->w_o, m.QD, ws.gemm_ws, ws.gemm_ws_bytes, st));

  // ---- adaLN: mod = silu(cond) W_ada^T + b_ada
  if (m.ada) {
    const long nmod = (long)S * 6 * d;
    BM_RETURN_IF(cast_from_f32(dt, ws.dmod, ws.dmod_e, nmod, st));
    BM_RETURN_IF(silu_forward(dt, cond, ws.sc, (long)S * d, st));
    BM_RETURN_IF(gemm(GEMM_TN, dt, 6 * d, d, S, ws.dmod_e, 6 * d, ws.sc, d, grads->w_ada, d, none,
                      ws.gemm_ws, ws.gemm_ws_bytes, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st); BM_RETURN_IF(colsum_accumulate(dt, ws.dmod_e, 6 * d, S, 6 * d, (float*)grads->b_ada, ws.colsum_ws, st)); }
    // d silu(cond) = dmod W_ada: a few rows against a long reduction, so it runs as a weight-gradient
    // style product on the transposed dmod (rows padded to 8), whose k range splits over the chip
    const int S8 = (int)align_up(S, 8);
    BM_RETURN_IF(cast_transpose_from_f32(dt, ws.dmod, ws.dmod_t, S, 6 * d, S8, st));
    BM_RETURN_IF(fill_zero(ws.dsc, (size_t)S8 * d * sizeof(float), st));
    BM_RETURN_IF(gemm(GEMM_TN, dt, S8, d, 6 * d, ws.dmod_t, S8, w->w_ada, d, ws.dsc, d, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
    BM_RETURN_IF(silu_backward_f32(dt, cond, ws.dsc, dcond, (long)S * d, st));
  }
  return BM_OK;
}
