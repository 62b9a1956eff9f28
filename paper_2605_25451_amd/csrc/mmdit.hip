// bm_mmdit_sizes / bm_mmdit_forward / bm_mmdit_backward: the two-stream (text / image) adaLN
// block with joint attention (generator of Sec. 4.1, read as the two-stream block of the
// multimodal diffusion transformer literature).
//
// Every per-token operator runs once per stream on that stream's packed rows with that
// stream's weights, through the same norm / GEMM / activation kernels as the single-stream
// block.  Only attention sees both streams: q, k, v rows are moved into the joint order
// [text tokens ; image tokens] of every sample (the optional RMS normalisation of q and k over
// head_dim rides on that move), the packed variable-length attention kernels run once over the
// joint sequences, and the output rows are moved back.  jpos_s[r] is the joint row of row r of
// stream s; it is rebuilt from the two cu arrays in both passes instead of being saved.
#include "common.h"
#include "../../include/bigmac_mmdit.h"

#include <vector>

namespace bm {

namespace {

struct MDims {
  int Ts[2], T, Tmax, S, d, H, dh, F, QD, QKV;
  size_t es;
  int qk_norm;
};

MDims make_mdims(const bm_mmdit_desc& c, int Tt, int Ti, int S) {
  MDims m;
  m.Ts[0] = Tt; m.Ts[1] = Ti; m.T = Tt + Ti; m.Tmax = Tt > Ti ? Tt : Ti; m.S = S;
  m.d = c.block.hidden; m.H = c.block.n_q_heads; m.dh = c.block.head_dim; m.F = c.block.mlp_hidden;
  m.QD = m.H * m.dh; m.QKV = 3 * m.QD;
  m.es = elt_size(c.block.dtype);
  m.qk_norm = c.qk_norm;
  return m;
}

struct StreamSaved {
  float *stats1, *stats2, *mod;
  char *qkv_raw, *o, *x1, *up, *attn, *m;
};

struct MSaved {
  StreamSaved s[2];
  char *qkv_j, *o_j;
  float* lse;
  size_t bytes;
};

MSaved layout_saved(const MDims& m, void* base) {
  Arena a(base);
  MSaved v;
  for (int s = 0; s < 2; ++s) {
    const size_t T = m.Ts[s];
    StreamSaved& q = v.s[s];
    q.stats1 = a.take<float>(2 * T * sizeof(float));
    q.stats2 = a.take<float>(2 * T * sizeof(float));
    q.mod = a.take<float>((size_t)m.S * 6 * m.d * sizeof(float));
    q.qkv_raw = m.qk_norm ? a.take<char>(T * m.QKV * m.es) : nullptr;
    q.o = a.take<char>(T * m.QD * m.es);
    q.x1 = a.take<char>(T * m.d * m.es);
    q.up = a.take<char>(T * m.F * m.es);
    q.attn = a.take<char>(T * m.d * m.es);
    q.m = a.take<char>(T * m.d * m.es);
  }
  v.qkv_j = a.take<char>((size_t)m.T * m.QKV * m.es);
  v.o_j = a.take<char>((size_t)m.T * m.QD * m.es);
  v.lse = a.take<float>((size_t)m.H * m.T * sizeof(float));
  v.bytes = a.off;
  return v;
}

// index tables shared by both passes
struct Tables {
  int32_t* tok_seq[2];
  int32_t* jpos[2];
  int32_t* jcu;
};

void take_tables(Arena& a, const MDims& m, Tables& t) {
  for (int s = 0; s < 2; ++s) {
    t.tok_seq[s] = a.take<int32_t>((size_t)m.Ts[s] * sizeof(int32_t));
    t.jpos[s] = a.take<int32_t>((size_t)m.Ts[s] * sizeof(int32_t));
  }
  t.jcu = a.take<int32_t>((size_t)(m.S + 1) * sizeof(int32_t));
}

struct MFwd {
  Tables tb;
  char *sc, *h, *qkv, *a;
  size_t bytes;
};

MFwd layout_fwd(const MDims& m, void* base) {
  Arena a(base);
  MFwd w;
  take_tables(a, m, w.tb);
  const size_t R = m.Tmax;
  w.sc = a.take<char>((size_t)m.S * m.d * m.es);
  w.h = a.take<char>(R * m.d * m.es);
  w.qkv = m.qk_norm ? nullptr : a.take<char>(R * m.QKV * m.es);
  w.a = a.take<char>(R * m.F * m.es);
  w.bytes = a.off;
  return w;
}

struct MBwd {
  Tables tb;
  char *dx1[2];                 // gradient at the mid-block residual, per stream, kept across the attention
  float* dmod[2];               // [S, 6d] per stream
  float* dsc[2];                // [S, d] per stream
  char *d_o_j, *dqkv_j;         // joint order
  char *a, *dup, *da, *h, *dh, *dgated, *d_o, *dqkv, *dmod_e, *dmod_t, *sc;   // per-stream temporaries, reused
  float* gain_part;             // per-workgroup partial sums of the q/k gain gradients
  char *attn_ws, *norm_ws, *colsum_ws, *gemm_ws;
  size_t attn_ws_bytes, gemm_ws_bytes;
  size_t bytes;
};

constexpr int QKN_BLOCKS = 512;     // workgroups per (q | k | v) plane of the q/k-norm backward

size_t max_gemm_scratch(const MDims& m, int dtype) {
  size_t b = 0, v;
  for (int s = 0; s < 2; ++s) {
    const int T = m.Ts[s];
    v = gemm_scratch_bytes(GEMM_TN, m.d, m.F, T, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_TN, m.F, m.d, T, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_TN, m.d, m.QD, T, dtype); b = v > b ? v : b;
    v = gemm_scratch_bytes(GEMM_TN, m.QKV, m.d, T, dtype); b = v > b ? v : b;
  }
  v = gemm_scratch_bytes(GEMM_TN, 6 * m.d, m.d, m.S, dtype); b = v > b ? v : b;
  v = gemm_scratch_bytes(GEMM_TN, (int)align_up(m.S, 8), m.d, 6 * m.d, dtype); b = v > b ? v : b;
  return b;
}

MBwd layout_bwd(const MDims& m, int dtype, void* base) {
  Arena a(base);
  MBwd w;
  take_tables(a, m, w.tb);
  for (int s = 0; s < 2; ++s) {
    w.dx1[s] = a.take<char>((size_t)m.Ts[s] * m.d * m.es);
    w.dmod[s] = a.take<float>((size_t)m.S * 6 * m.d * sizeof(float));
    w.dsc[s] = a.take<float>(align_up(m.S, 8) * m.d * sizeof(float));
  }
  w.d_o_j = a.take<char>((size_t)m.T * m.QD * m.es);
  w.dqkv_j = a.take<char>((size_t)m.T * m.QKV * m.es);
  const size_t R = m.Tmax;
  w.a = a.take<char>(R * m.F * m.es);
  w.dup = a.take<char>(R * m.F * m.es);
  w.da = a.take<char>(R * m.F * m.es);
  w.h = a.take<char>(R * m.d * m.es);
  w.dh = a.take<char>(R * m.d * m.es);
  w.dgated = a.take<char>(R * m.d * m.es);
  w.d_o = a.take<char>(R * m.QD * m.es);
  w.dqkv = a.take<char>(R * m.QKV * m.es);
  w.dmod_e = a.take<char>((size_t)m.S * 6 * m.d * m.es);
  w.dmod_t = a.take<char>(align_up(m.S, 8) * 6 * m.d * m.es);
  w.sc = a.take<char>((size_t)m.S * m.d * m.es);
  w.gain_part = a.take<float>((size_t)QKN_BLOCKS * 2 * m.dh * sizeof(float));
  w.attn_ws_bytes = attention_backward_scratch_bytes(m.H, m.H, m.dh, m.T);
  w.attn_ws = a.take<char>(w.attn_ws_bytes);
  w.norm_ws = a.take<char>(norm_backward_scratch_bytes(m.Tmax, m.d));
  int widest = m.F > m.QKV ? m.F : m.QKV;
  if (6 * m.d > widest) widest = 6 * m.d;
  w.colsum_ws = a.take<char>(colsum_scratch_bytes(m.Tmax > QKN_BLOCKS ? m.Tmax : QKN_BLOCKS, widest));
  w.gemm_ws_bytes = max_gemm_scratch(m, dtype);
  w.gemm_ws = a.take<char>(w.gemm_ws_bytes);
  w.bytes = a.off;
  return w;
}

// ------------------------------------------------------------------ index kernels
// joint row of every row of one stream: the sample's joint sequence is [text ; image]
__global__ void joint_pos_kernel(const int32_t* __restrict__ cu_own, const int32_t* __restrict__ cu_other,
                                 const int32_t* __restrict__ tok_seq, int rows, int is_image,
                                 int32_t* __restrict__ jpos) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  const int b = tok_seq[r];
  int base = cu_own[b] + cu_other[b];
  if (is_image) base += cu_other[b + 1] - cu_other[b];
  jpos[r] = base + (r - cu_own[b]);
}

__global__ void joint_cu_kernel(const int32_t* __restrict__ cu_a, const int32_t* __restrict__ cu_b, int n,
                                int32_t* __restrict__ jcu) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) jcu[i] = cu_a[i] + cu_b[i];
}

bm_status build_tables(const MDims& m, const Tables& tb, const int32_t* const cu_dev[2], hipStream_t st) {
  for (int s = 0; s < 2; ++s) {
    BM_RETURN_IF(launch_tok_seq(cu_dev[s], m.S, m.Ts[s], tb.tok_seq[s], st));
    hipLaunchKernelGGL(joint_pos_kernel, dim3(cdiv(m.Ts[s], 256)), dim3(256), 0, st, cu_dev[s], cu_dev[1 - s],
                       tb.tok_seq[s], m.Ts[s], s, tb.jpos[s]);
  }
  hipLaunchKernelGGL(joint_cu_kernel, dim3(cdiv(m.S + 1, 256)), dim3(256), 0, st, cu_dev[0], cu_dev[1], m.S + 1,
                     tb.jcu);
  BM_CHECK_LAUNCH("mmdit tables");
  return BM_OK;
}

// ------------------------------------------------------------------ q/k RMS normalisation
// A group of LP lanes (power of two, <= 64) owns one head vector of one row; lane c of the group
// holds elements [c*VEC, c*VEC+VEC) when c < dh/VEC.  blockIdx.y selects the plane: 0 q, 1 k, 2 v.

template <int LP>
__device__ inline float group_sum(float v) {
#pragma unroll
  for (int off = LP / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}

// forward: qkv_j[jpos[r], plane, head, :] = plane < 2 ? raw / rms(raw) * gain_plane : raw
template <typename T, int LP>
__global__ __launch_bounds__(256) void qk_norm_fwd_kernel(const T* __restrict__ raw, const int32_t* __restrict__ jpos,
                                                          const T* __restrict__ gq, const T* __restrict__ gk,
                                                          T* __restrict__ out, int rows, int H, int dh, float eps) {
  constexpr int VEC = Elt<T>::VEC;
  constexpr int GROUPS = 256 / LP;
  const int plane = blockIdx.y;
  const int lane_c = threadIdx.x % LP;
  const bool live = lane_c * VEC < dh;
  const long items = (long)rows * H;
  const int QD = H * dh;
  float g[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) g[e] = 1.f;
  if (plane < 2 && live) load16((plane == 0 ? gq : gk) + lane_c * VEC, g);
  for (long it = (long)blockIdx.x * GROUPS + threadIdx.x / LP; it < items; it += (long)gridDim.x * GROUPS) {
    const int r = (int)(it / H), hd = (int)(it % H);
    const size_t col = (size_t)plane * QD + (size_t)hd * dh + lane_c * VEC;
    float v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = 0.f;
    if (live) load16(raw + (size_t)r * 3 * QD + col, v);
    if (plane < 2) {
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) ss += v[e] * v[e];
      ss = group_sum<LP>(ss);
      const float rs = rsqrtf(ss / (float)dh + eps);
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = v[e] * rs * g[e];
    }
    if (live) store16(out + (size_t)jpos[r] * 3 * QD + col, v);
  }
}

// backward: dqkv[r] = d(raw) from dqkv_j[jpos[r]]; per-workgroup partial sums of the gain
// gradients go to part[blockIdx.x][plane][dh] (every workgroup writes its slot, zeros included)
template <typename T, int LP>
__global__ __launch_bounds__(256) void qk_norm_bwd_kernel(const T* __restrict__ dout_j, const T* __restrict__ raw,
                                                          const int32_t* __restrict__ jpos,
                                                          const T* __restrict__ gq, const T* __restrict__ gk,
                                                          T* __restrict__ dqkv, float* __restrict__ part, int rows,
                                                          int H, int dh, float eps) {
  constexpr int VEC = Elt<T>::VEC;
  constexpr int GROUPS = 256 / LP;
  __shared__ float sm[GROUPS][LP * VEC];
  const int plane = blockIdx.y;
  const int lane_c = threadIdx.x % LP, grp = threadIdx.x / LP;
  const bool live = lane_c * VEC < dh;
  const long items = (long)rows * H;
  const int QD = H * dh;
  float g[VEC], dg[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { g[e] = 1.f; dg[e] = 0.f; }
  if (plane < 2 && live) load16((plane == 0 ? gq : gk) + lane_c * VEC, g);
  for (long it = (long)blockIdx.x * GROUPS + grp; it < items; it += (long)gridDim.x * GROUPS) {
    const int r = (int)(it / H), hd = (int)(it % H);
    const size_t col = (size_t)plane * QD + (size_t)hd * dh + lane_c * VEC;
    float dv[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) dv[e] = 0.f;
    if (live) load16(dout_j + (size_t)jpos[r] * 3 * QD + col, dv);
    if (plane < 2) {
      float t[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) t[e] = 0.f;
      if (live) load16(raw + (size_t)r * 3 * QD + col, t);
      float ss = 0.f, dot = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) { ss += t[e] * t[e]; dot += dv[e] * g[e] * t[e]; }
      ss = group_sum<LP>(ss);
      dot = group_sum<LP>(dot);
      const float rs = rsqrtf(ss / (float)dh + eps);
      const float k = rs * rs * rs * dot / (float)dh;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        dg[e] += dv[e] * t[e] * rs;
        dv[e] = rs * dv[e] * g[e] - t[e] * k;
      }
    }
    if (live) store16(dqkv + (size_t)r * 3 * QD + col, dv);
  }
  if (plane < 2) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) sm[grp][lane_c * VEC + e] = dg[e];
    __syncthreads();
    if ((int)threadIdx.x < dh) {
      float s = 0.f;
      for (int q = 0; q < GROUPS; ++q) s += sm[q][threadIdx.x];
      part[((size_t)blockIdx.x * 2 + plane) * dh + threadIdx.x] = s;
    }
  }
}

int lanes_per_head(int dh, int vec) {
  int lp = 1;
  while (lp * vec < dh) lp *= 2;
  return lp;
}

int qkn_blocks(long items, int lp) {
  long want = (items + 256 / lp - 1) / (256 / lp);
  return (int)(want < QKN_BLOCKS ? (want < 1 ? 1 : want) : QKN_BLOCKS);
}

bm_status qk_norm_forward(int dtype, const void* raw, const int32_t* jpos, const void* gq, const void* gk,
                          void* out, int rows, int H, int dh, float eps, hipStream_t st) {
  if (rows == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  const int lp = lanes_per_head(dh, vec);
  dim3 grid(qkn_blocks((long)rows * H, lp), 3), block(256);
#define BM_L(TT, LPV)                                                                                         \
  hipLaunchKernelGGL((qk_norm_fwd_kernel<TT, LPV>), grid, block, 0, st, (const TT*)raw, jpos, (const TT*)gq,  \
                     (const TT*)gk, (TT*)out, rows, H, dh, eps)
#define BM_D(TT)                                                                                              \
  switch (lp) {                                                                                               \
    case 1: BM_L(TT, 1); break; case 2: BM_L(TT, 2); break; case 4: BM_L(TT, 4); break;                       \
    case 8: BM_L(TT, 8); break; case 16: BM_L(TT, 16); break; case 32: BM_L(TT, 32); break;                   \
    default: set_error("q/k norm: head_dim %d unsupported", dh); return BM_ERR_UNSUPPORTED;                   \
  }
  if (dtype == BM_DTYPE_BF16) { BM_D(bf16_t) } else { BM_D(float) }
#undef BM_L
#undef BM_D
  BM_CHECK_LAUNCH("qk_norm_fwd");
  return BM_OK;
}

bm_status qk_norm_backward(int dtype, const void* dout_j, const void* raw, const int32_t* jpos, const void* gq,
                           const void* gk, void* dqkv, float* part, float* dgq, float* dgk, void* colsum_ws,
                           int rows, int H, int dh, float eps, hipStream_t st) {
  if (rows == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  const int lp = lanes_per_head(dh, vec);
  const int blocks = qkn_blocks((long)rows * H, lp);
  dim3 grid(blocks, 3), block(256);
#define BM_L(TT, LPV)                                                                                          \
  hipLaunchKernelGGL((qk_norm_bwd_kernel<TT, LPV>), grid, block, 0, st, (const TT*)dout_j, (const TT*)raw,     \
                     jpos, (const TT*)gq, (const TT*)gk, (TT*)dqkv, part, rows, H, dh, eps)
#define BM_D(TT)                                                                                               \
  switch (lp) {                                                                                                \
    case 1: BM_L(TT, 1); break; case 2: BM_L(TT, 2); break; case 4: BM_L(TT, 4); break;                        \
    case 8: BM_L(TT, 8); break; case 16: BM_L(TT, 16); break; case 32: BM_L(TT, 32); break;                    \
    default: set_error("q/k norm: head_dim %d unsupported", dh); return BM_ERR_UNSUPPORTED;                    \
  }
  if (dtype == BM_DTYPE_BF16) { BM_D(bf16_t) } else { BM_D(float) }
#undef BM_L
#undef BM_D
  BM_CHECK_LAUNCH("qk_norm_bwd");
  // fixed-order sum over workgroups, added to the gradients
  BM_RETURN_IF(colsum_accumulate(BM_DTYPE_FP32, part, 2 * dh, blocks, dh, dgq, colsum_ws, st));
  BM_RETURN_IF(colsum_accumulate(BM_DTYPE_FP32, part + dh, 2 * dh, blocks, dh, dgk, colsum_ws, st));
  return BM_OK;
}

// ------------------------------------------------------------------ argument checks
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

#define NEED_PTR(p)                                                          \
  do {                                                                       \
    BM_ARG_CHECK((p) != nullptr, #p " is NULL");                             \
    BM_ARG_CHECK(aligned16(p), #p " is not 16-byte aligned");                \
  } while (0)

bm_status check_mdesc(const bm_mmdit_desc* c) {
  BM_ARG_CHECK(c != nullptr, "desc is NULL");
  // the single-stream checks (sizes, head_dim, dtype, vector widths)
  size_t a, b;
  BM_RETURN_IF(bm_block_sizes(&c->block, 1, 1, 1, &a, &b));
  const bm_block_desc& k = c->block;
  if (k.norm != BM_NORM_ADALN || k.act != BM_ACT_GELU || k.mask != BM_MASK_BIDIRECTIONAL || k.rope ||
      !k.linear_bias || k.n_experts != 0 || k.n_q_heads != k.n_kv_heads) {
    set_error("mmdit desc: needs norm = adaLN, act = GELU, bidirectional mask, no RoPE, linear_bias = 1, "
              "no experts, n_q_heads = n_kv_heads");
    return BM_ERR_UNSUPPORTED;
  }
  BM_ARG_CHECK(c->qk_norm == 0 || c->qk_norm == 1, "mmdit desc: qk_norm %d", c->qk_norm);
  BM_ARG_CHECK(!c->qk_norm || c->qk_norm_eps >= 0.f, "mmdit desc: qk_norm_eps negative");
  return BM_OK;
}

bm_status check_stream_params(const bm_mmdit_desc& c, const bm_mmdit_params* p, const char* what) {
  BM_ARG_CHECK(p != nullptr, "%s is NULL", what);
  for (int s = 0; s < 2; ++s) {
    const bm_block_params& q = p->stream[s];
#define NEED(f)                                                                                       \
  do {                                                                                                \
    BM_ARG_CHECK(q.f != nullptr, "%s.stream[%d].%s is NULL", what, s, #f);                            \
    BM_ARG_CHECK(aligned16(q.f), "%s.stream[%d].%s is not 16-byte aligned", what, s, #f);             \
  } while (0)
    NEED(w_qkv); NEED(b_qkv); NEED(w_o); NEED(b_o); NEED(w_up); NEED(b_up); NEED(w_down); NEED(b_down);
    NEED(w_ada); NEED(b_ada);
#undef NEED
    if (c.qk_norm) {
      BM_ARG_CHECK(p->q_norm_g[s] && p->k_norm_g[s], "%s: q/k norm gains of stream %d are NULL", what, s);
      BM_ARG_CHECK(aligned16(p->q_norm_g[s]) && aligned16(p->k_norm_g[s]),
                   "%s: q/k norm gains of stream %d are not 16-byte aligned", what, s);
    }
  }
  return BM_OK;
}

// both cu arrays on the host: validity, then the joint offsets
bm_status check_streams(const int32_t* const cu_dev[2], const int32_t* const cu_host[2], int S,
                        std::vector<int32_t>& jcu, int* Ts, int* max_joint) {
  BM_ARG_CHECK(S >= 1, "S must be positive (S=%d)", S);
  for (int s = 0; s < 2; ++s) {
    BM_ARG_CHECK(cu_dev[s] && cu_host[s], "cu_seqlens pointers of stream %d must not be NULL", s);
    BM_ARG_CHECK(cu_host[s][0] == 0, "stream %d: cu_seqlens[0] = %d, expected 0", s, cu_host[s][0]);
    for (int b = 0; b < S; ++b)
      BM_ARG_CHECK(cu_host[s][b + 1] - cu_host[s][b] >= 1, "stream %d: sample %d has length %d (must be >= 1)", s,
                   b, cu_host[s][b + 1] - cu_host[s][b]);
    Ts[s] = cu_host[s][S];
  }
  BM_ARG_CHECK((long)Ts[0] + Ts[1] <= (long)INT32_MAX / 2, "joint token count too large");
  jcu.resize(S + 1);
  *max_joint = 0;
  for (int b = 0; b <= S; ++b) {
    jcu[b] = cu_host[0][b] + cu_host[1][b];
    if (b && jcu[b] - jcu[b - 1] > *max_joint) *max_joint = jcu[b] - jcu[b - 1];
  }
  return BM_OK;
}

// no tensor of a call may reach 2^31 elements (joint rows x the widest row), as for the single-stream block
bm_status check_mextent(const bm_mmdit_desc& c, long T_text, long T_img) {
  const long d = c.block.hidden, qkv = 3L * c.block.n_q_heads * c.block.head_dim, up = c.block.mlp_hidden;
  long widest = qkv > up ? qkv : up;
  if (d > widest) widest = d;
  BM_ARG_CHECK((T_text + T_img) * widest < (1L << 31),
               "%ld joint rows x %ld columns reach 2^31 elements: split the pack", T_text + T_img, widest);
  return BM_OK;
}

NormArgs ada_norm_args(const bm_block_desc& c, int T, int which, const float* mod, const int32_t* tok_seq) {
  NormArgs n;
  n.dtype = c.dtype; n.kind = BM_NORM_ADALN; n.T = T; n.d = c.hidden; n.eps = c.norm_eps;
  n.mod = mod; n.ld_mod = 6 * c.hidden;
  n.shift_off = which == 1 ? 0 : 3 * c.hidden;
  n.scale_off = which == 1 ? c.hidden : 4 * c.hidden;
  n.tok_seq = tok_seq;
  return n;
}

AttnArgs joint_attn_args(const bm_block_desc& c, const MDims& m, const char* qkv_j, const int32_t* jcu_dev,
                         const int32_t* jcu_host, int max_joint) {
  AttnArgs at;
  at.dtype = c.dtype; at.causal = 0; at.Hq = m.H; at.Hkv = m.H; at.dh = m.dh;
  at.q = qkv_j; at.k = qkv_j + (size_t)m.QD * m.es; at.v = qkv_j + (size_t)2 * m.QD * m.es;
  at.ld_qkv = m.QKV; at.cu_dev = jcu_dev; at.cu_host = jcu_host; at.S = m.S; at.T = m.T;
  at.max_seqlen = max_joint;
  return at;
}

}  // namespace

}  // namespace bm

using namespace bm;

extern "C" bm_status bm_mmdit_sizes(const bm_mmdit_desc* desc, int32_t T_text, int32_t T_img, int32_t S,
                                    size_t* saved_bytes, size_t* scratch_bytes) {
  BM_RETURN_IF(check_mdesc(desc));
  BM_ARG_CHECK(S >= 1 && T_text >= S && T_img >= S, "bm_mmdit_sizes: bad T_text=%d T_img=%d S=%d", T_text, T_img, S);
  BM_ARG_CHECK(saved_bytes && scratch_bytes, "bm_mmdit_sizes: output pointers are NULL");
  BM_RETURN_IF(check_mextent(*desc, T_text, T_img));
  MDims m = make_mdims(*desc, T_text, T_img, S);
  *saved_bytes = layout_saved(m, nullptr).bytes;
  size_t f = layout_fwd(m, nullptr).bytes, b = layout_bwd(m, desc->block.dtype, nullptr).bytes;
  *scratch_bytes = f > b ? f : b;
  return BM_OK;
}

extern "C" bm_status bm_mmdit_forward(const bm_mmdit_desc* desc, const bm_mmdit_params* w,
                                      const void* x_text, const void* x_img,
                                      const int32_t* cu_text_dev, const int32_t* cu_text_host,
                                      const int32_t* cu_img_dev, const int32_t* cu_img_host, int32_t S,
                                      const void* cond, void* y_text, void* y_img, void* saved, void* scratch,
                                      size_t scratch_bytes, void* hip_stream) {
  BM_RETURN_IF(check_mdesc(desc));
  const bm_block_desc& c = desc->block;
  const int32_t* const cu_dev[2] = {cu_text_dev, cu_img_dev};
  const int32_t* const cu_host[2] = {cu_text_host, cu_img_host};
  std::vector<int32_t> jcu_host;
  int Ts[2], max_joint;
  BM_RETURN_IF(check_streams(cu_dev, cu_host, S, jcu_host, Ts, &max_joint));
  BM_RETURN_IF(check_mextent(*desc, Ts[0], Ts[1]));
  BM_RETURN_IF(check_stream_params(*desc, w, "w"));
  NEED_PTR(x_text); NEED_PTR(x_img); NEED_PTR(y_text); NEED_PTR(y_img); NEED_PTR(cond); NEED_PTR(saved);
  NEED_PTR(scratch);
  BM_ARG_CHECK(x_text != y_text && x_img != y_img, "y must not alias x");
  const void* const x[2] = {x_text, x_img};
  void* const y[2] = {y_text, y_img};
  MDims m = make_mdims(*desc, Ts[0], Ts[1], S);
  MFwd ws = layout_fwd(m, scratch);
  if (ws.bytes > scratch_bytes) {
    set_error("forward needs %zu scratch bytes, got %zu", ws.bytes, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  MSaved sv = layout_saved(m, saved);
  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c.dtype, d = m.d;

  BM_RETURN_IF(build_tables(m, ws.tb, cu_dev, st));
  BM_RETURN_IF(silu_forward(dt, cond, ws.sc, (long)S * d, st));

  // ---- per stream: modulation, norm 1, qkv, move into the joint order
  for (int s = 0; s < 2; ++s) {
    const bm_block_params& p = w->stream[s];
    const int T = m.Ts[s];
    {
      GemmEpilogue e; e.bias = p.b_ada; e.out_fp32 = 1;
      BM_RETURN_IF(gemm(GEMM_NT, dt, S, 6 * d, d, ws.sc, d, p.w_ada, d, sv.s[s].mod, 6 * d, e, nullptr, 0, st));
    }
    { ProfScope _p(PROF_NORM, 2.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(norm_forward(ada_norm_args(c, T, 1, sv.s[s].mod, ws.tb.tok_seq[s]), x[s], ws.h, sv.s[s].stats1, 1, st)); }
    char* qkv = m.qk_norm ? sv.s[s].qkv_raw : ws.qkv;
    {
      GemmEpilogue e; e.bias = p.b_qkv;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.QKV, d, ws.h, d, p.w_qkv, d, qkv, m.QKV, e, nullptr, 0, st));
    }
    ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * m.QKV * (double)m.es, st);
    if (m.qk_norm)
      BM_RETURN_IF(qk_norm_forward(dt, qkv, ws.tb.jpos[s], w->q_norm_g[s], w->k_norm_g[s], sv.qkv_j, T, m.H, m.dh,
                                   desc->qk_norm_eps, st));
    else
      BM_RETURN_IF(row_scatter(dt, qkv, ws.tb.jpos[s], sv.qkv_j, T, m.QKV, st));
  }

  // ---- joint attention
  AttnArgs at = joint_attn_args(c, m, sv.qkv_j, ws.tb.jcu, jcu_host.data(), max_joint);
  BM_RETURN_IF(attention_forward(at, sv.o_j, sv.lse, st));

  // ---- per stream: output projection, gated residual, MLP
  for (int s = 0; s < 2; ++s) {
    const bm_block_params& p = w->stream[s];
    const StreamSaved& q = sv.s[s];
    const int T = m.Ts[s];
    const int32_t* tok = ws.tb.tok_seq[s];
    { ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * m.QD * (double)m.es, st);
      BM_RETURN_IF(row_gather(dt, sv.o_j, ws.tb.jpos[s], q.o, T, m.QD, st)); }
    {
      GemmEpilogue e; e.bias = p.b_o;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, d, m.QD, q.o, m.QD, p.w_o, m.QD, q.attn, d, e, nullptr, 0, st));
    }
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(gate_mul(dt, q.attn, q.mod + 2 * d, 6 * d, tok, x[s], q.x1, T, d, st)); }
    { ProfScope _p(PROF_NORM, 2.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(norm_forward(ada_norm_args(c, T, 2, q.mod, tok), q.x1, ws.h, q.stats2, 1, st)); }
    {
      GemmEpilogue e; e.bias = p.b_up;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, m.F, d, ws.h, d, p.w_up, d, q.up, m.F, e, nullptr, 0, st));
    }
    { ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * m.F * (double)m.es, st);
      BM_RETURN_IF(act_forward(dt, BM_ACT_GELU, q.up, ws.a, T, m.F, st)); }
    {
      GemmEpilogue e; e.bias = p.b_down;
      BM_RETURN_IF(gemm(GEMM_NT, dt, T, d, m.F, ws.a, m.F, p.w_down, m.F, q.m, d, e, nullptr, 0, st));
    }
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(gate_mul(dt, q.m, q.mod + 5 * d, 6 * d, tok, q.x1, y[s], T, d, st)); }
  }
  return BM_OK;
}

extern "C" bm_status bm_mmdit_backward(const bm_mmdit_desc* desc, const bm_mmdit_params* w,
                                       const void* x_text, const void* x_img,
                                       const void* dy_text, const void* dy_img,
                                       const int32_t* cu_text_dev, const int32_t* cu_text_host,
                                       const int32_t* cu_img_dev, const int32_t* cu_img_host, int32_t S,
                                       const void* cond, const void* saved, void* dx_text, void* dx_img,
                                       const bm_mmdit_params* grads, void* dcond, void* scratch,
                                       size_t scratch_bytes, void* hip_stream) {
  BM_RETURN_IF(check_mdesc(desc));
  const bm_block_desc& c = desc->block;
  const int32_t* const cu_dev[2] = {cu_text_dev, cu_img_dev};
  const int32_t* const cu_host[2] = {cu_text_host, cu_img_host};
  std::vector<int32_t> jcu_host;
  int Ts[2], max_joint;
  BM_RETURN_IF(check_streams(cu_dev, cu_host, S, jcu_host, Ts, &max_joint));
  BM_RETURN_IF(check_mextent(*desc, Ts[0], Ts[1]));
  BM_RETURN_IF(check_stream_params(*desc, w, "w"));
  BM_RETURN_IF(check_stream_params(*desc, grads, "grads"));
  NEED_PTR(x_text); NEED_PTR(x_img); NEED_PTR(dy_text); NEED_PTR(dy_img); NEED_PTR(dx_text); NEED_PTR(dx_img);
  NEED_PTR(cond); NEED_PTR(dcond); NEED_PTR(saved); NEED_PTR(scratch);
  BM_ARG_CHECK(dx_text != dy_text && dx_text != x_text && dx_img != dy_img && dx_img != x_img,
               "dx must not alias dy or x");
  const void* const x[2] = {x_text, x_img};
  const void* const dy[2] = {dy_text, dy_img};
  void* const dx[2] = {dx_text, dx_img};
  MDims m = make_mdims(*desc, Ts[0], Ts[1], S);
  MBwd ws = layout_bwd(m, c.dtype, scratch);
  if (ws.bytes > scratch_bytes) {
    set_error("backward needs %zu scratch bytes, got %zu", ws.bytes, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  MSaved sv = layout_saved(m, const_cast<void*>(saved));
  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c.dtype, d = m.d;
  const GemmEpilogue none;

  BM_RETURN_IF(build_tables(m, ws.tb, cu_dev, st));

  // ---- per stream: MLP half and output projection, down to the attention output gradient
  for (int s = 0; s < 2; ++s) {
    const bm_block_params& p = w->stream[s];
    const bm_block_params& g = grads->stream[s];
    const StreamSaved& q = sv.s[s];
    const int T = m.Ts[s];
    const int32_t* tok = ws.tb.tok_seq[s];
    float* dmod = ws.dmod[s];
    // y = x1 + g2 * m,  m = a W_down^T + b_down
    { ProfScope _p(PROF_ELEMENTWISE, 3.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(segment_gate(dt, dy[s], q.m, q.mod + 5 * d, 6 * d, ws.dgated, cu_dev[s], S, d, dmod + 5 * d, 6 * d,
                                ws.norm_ws, st)); }
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, m.F, d, ws.dgated, d, p.w_down, m.F, ws.da, m.F, none, nullptr, 0, st));
    { ProfScope _p(PROF_ELEMENTWISE, (double)T * 4.0 * m.F * (double)m.es, st);
      BM_RETURN_IF(act_backward(dt, BM_ACT_GELU, q.up, ws.da, ws.dup, ws.a, (float*)g.b_up, ws.colsum_ws, T, m.F, st)); }
    BM_RETURN_IF(gemm(GEMM_TN, dt, d, m.F, T, ws.dgated, d, ws.a, m.F, g.w_down, m.F, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(colsum_accumulate(dt, ws.dgated, d, T, d, (float*)g.b_down, ws.colsum_ws, st)); }
    // up = h2 W_up^T + b_up,  h2 = LN0(x1)(1 + scale2) + shift2
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, d, m.F, ws.dup, m.F, p.w_up, d, ws.dh, d, none, nullptr, 0, st));
    { ProfScope _p(PROF_NORM, 5.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(norm_backward(ada_norm_args(c, T, 2, q.mod, tok), q.x1, q.stats2, ws.dh, dy[s], ws.dx1[s], ws.h,
                                 nullptr, nullptr, nullptr, nullptr, dmod, cu_dev[s], S, ws.norm_ws, st)); }
    BM_RETURN_IF(gemm(GEMM_TN, dt, m.F, d, T, ws.dup, m.F, ws.h, d, g.w_up, d, none, ws.gemm_ws, ws.gemm_ws_bytes, st));
    // x1 = x + g1 * attn,  attn = o W_o^T + b_o
    { ProfScope _p(PROF_ELEMENTWISE, 3.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(segment_gate(dt, ws.dx1[s], q.attn, q.mod + 2 * d, 6 * d, ws.dgated, cu_dev[s], S, d, dmod + 2 * d,
                                6 * d, ws.norm_ws, st)); }
    BM_RETURN_IF(gemm(GEMM_TN, dt, d, m.QD, T, ws.dgated, d, q.o, m.QD, g.w_o, m.QD, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(colsum_accumulate(dt, ws.dgated, d, T, d, (float*)g.b_o, ws.colsum_ws, st)); }
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, m.QD, d, ws.dgated, d, p.w_o, m.QD, ws.d_o, m.QD, none, nullptr, 0, st));
    { ProfScope _p(PROF_ELEMENTWISE, 2.0 * T * m.QD * (double)m.es, st);
      BM_RETURN_IF(row_scatter(dt, ws.d_o, ws.tb.jpos[s], ws.d_o_j, T, m.QD, st)); }
  }

  // ---- joint attention
  AttnArgs at = joint_attn_args(c, m, sv.qkv_j, ws.tb.jcu, jcu_host.data(), max_joint);
  BM_RETURN_IF(attention_backward(at, sv.o_j, ws.d_o_j, sv.lse, ws.dqkv_j, ws.dqkv_j + (size_t)m.QD * m.es,
                                  ws.dqkv_j + (size_t)2 * m.QD * m.es, m.QKV, ws.attn_ws, ws.attn_ws_bytes, st));

  // ---- per stream: back out of the joint order, qkv projection, norm 1, modulation
  BM_RETURN_IF(silu_forward(dt, cond, ws.sc, (long)S * d, st));
  for (int s = 0; s < 2; ++s) {
    const bm_block_params& p = w->stream[s];
    const bm_block_params& g = grads->stream[s];
    const StreamSaved& q = sv.s[s];
    const int T = m.Ts[s];
    const int32_t* tok = ws.tb.tok_seq[s];
    float* dmod = ws.dmod[s];
    {
      ProfScope _p(PROF_ELEMENTWISE, (m.qk_norm ? 3.0 : 2.0) * T * m.QKV * (double)m.es, st);
      if (m.qk_norm)
        BM_RETURN_IF(qk_norm_backward(dt, ws.dqkv_j, q.qkv_raw, ws.tb.jpos[s], w->q_norm_g[s], w->k_norm_g[s],
                                      ws.dqkv, ws.gain_part, (float*)grads->q_norm_g[s], (float*)grads->k_norm_g[s],
                                      ws.colsum_ws, T, m.H, m.dh, desc->qk_norm_eps, st));
      else
        BM_RETURN_IF(row_gather(dt, ws.dqkv_j, ws.tb.jpos[s], ws.dqkv, T, m.QKV, st));
      BM_RETURN_IF(colsum_accumulate(dt, ws.dqkv, m.QKV, T, m.QKV, (float*)g.b_qkv, ws.colsum_ws, st));
    }
    BM_RETURN_IF(gemm(GEMM_NN, dt, T, d, m.QKV, ws.dqkv, m.QKV, p.w_qkv, d, ws.dh, d, none, nullptr, 0, st));
    { ProfScope _p(PROF_NORM, 5.0 * T * d * (double)m.es, st);
      BM_RETURN_IF(norm_backward(ada_norm_args(c, T, 1, q.mod, tok), x[s], q.stats1, ws.dh, ws.dx1[s], dx[s], ws.h,
                                 nullptr, nullptr, nullptr, nullptr, dmod, cu_dev[s], S, ws.norm_ws, st)); }
    BM_RETURN_IF(gemm(GEMM_TN, dt, m.QKV, d, T, ws.dqkv, m.QKV, ws.h, d, g.w_qkv, d, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
    // mod = silu(cond) W_ada^T + b_ada
    BM_RETURN_IF(cast_from_f32(dt, dmod, ws.dmod_e, (long)S * 6 * d, st));
    BM_RETURN_IF(gemm(GEMM_TN, dt, 6 * d, d, S, ws.dmod_e, 6 * d, ws.sc, d, g.w_ada, d, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
    { ProfScope _p(PROF_ELEMENTWISE, 0.0, st);
      BM_RETURN_IF(colsum_accumulate(dt, ws.dmod_e, 6 * d, S, 6 * d, (float*)g.b_ada, ws.colsum_ws, st)); }
    // d silu(cond) = dmod W_ada as a weight-gradient style product on the transposed dmod
    // (few rows, long reduction: the k range splits over the chip)
    const int S8 = (int)align_up(S, 8);
    BM_RETURN_IF(cast_transpose_from_f32(dt, dmod, ws.dmod_t, S, 6 * d, S8, st));
    BM_RETURN_IF(fill_zero(ws.dsc[s], (size_t)S8 * d * sizeof(float), st));
    BM_RETURN_IF(gemm(GEMM_TN, dt, S8, d, 6 * d, ws.dmod_t, S8, p.w_ada, d, ws.dsc[s], d, none, ws.gemm_ws,
                      ws.gemm_ws_bytes, st));
  }
  // both streams read the same conditioning rows
  BM_RETURN_IF(add_inplace(BM_DTYPE_FP32, ws.dsc[0], ws.dsc[1], (long)S * d, st));
  BM_RETURN_IF(silu_backward_f32(dt, cond, ws.dsc[0], dcond, (long)S * d, st));
  return BM_OK;
}
