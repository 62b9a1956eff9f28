// Routing, dispatch and combine kernels of the mixture-of-experts FFN.
//
// The paper's LLM backbone is a mixture-of-experts model (Sec. 4.1) and Sec. 3.3 names
// expert imbalance as a source of uneven operator times; it gives no arithmetic.  The
// reading built here: router logits = h W_r^T, probabilities = softmax over the experts,
// the k most probable experts are chosen (ties: lower index), their probabilities
// renormalised to sum 1 are the gates, no token is dropped.
//
// Dispatch layout.  The T*k routed rows are sorted by expert, token order inside an
// expert, and every expert's segment is padded to MOE_PAD rows, so a row block of the
// grouped GEMMs belongs to one expert.  The padded capacity T*k + E*(MOE_PAD-1), rounded
// up, is known on the host; everything data dependent (segment offsets, the row block ->
// expert table, the slot of each (token, choice)) stays on the device.  All counting is
// integer work in a fixed order, so the layout -- and with it every floating-point sum
// downstream -- is reproducible.
#include "common.h"

namespace bm {

namespace {

constexpr int MOE_MAX_E = 256;    // experts (4 logits per lane)
constexpr int MOE_MAX_K = 8;
constexpr int MOE_CHUNK = 256;    // tokens per workgroup in the counting kernels

// ---- router: softmax, top-k, gates (one wavefront per token) -------------------------
__global__ __launch_bounds__(256) void moe_route_kernel(const float* __restrict__ logits, int T, int E,
                                                        int k, float* __restrict__ probs,
                                                        int32_t* __restrict__ idx, float* __restrict__ gate) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  float v[4];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = i * 64 + lane;
    v[i] = e < E ? logits[(size_t)t * E + e] : -INFINITY;
    mx = fmaxf(mx, v[i]);
  }
  mx = wave_max(mx);
  float p[4], s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) { p[i] = (i * 64 + lane) < E ? expf(v[i] - mx) : 0.f; s += p[i]; }
  s = wave_sum(s);
  const float inv = 1.0f / s;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    p[i] *= inv;
    const int e = i * 64 + lane;
    if (e < E) probs[(size_t)t * E + e] = p[i];
  }
  // k rounds of (largest logit, lowest index); a chosen logit is retired to -inf
  float sel[MOE_MAX_K];
  int who[MOE_MAX_K];
  float ssum = 0.f;
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    sel[j] = 0.f; who[j] = 0;
    if (j >= k) continue;
    float bv = -INFINITY; int be = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = i * 64 + lane;
      if (e < E && v[i] > bv) { bv = v[i]; be = e; }      // ascending e: the lower index wins a tie
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off, WAVE);
      const int oe = __shfl_xor(be, off, WAVE);
      if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    // the owner retires it and everybody learns its probability
    float pw = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i * 64 + lane == be) { pw = p[i]; v[i] = -INFINITY; }
    pw = wave_sum(pw);
    sel[j] = pw; who[j] = be; ssum += pw;
  }
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
      if (j < k) {
        idx[(size_t)t * k + j] = who[j];
        gate[(size_t)t * k + j] = sel[j] / ssum;
      }
    }
  }
}

// ---- dispatch layout ---------------------------------------------------------------------
__global__ __launch_bounds__(MOE_CHUNK) void moe_count_kernel(const int32_t* __restrict__ idx, int T, int E,
                                                              int k, int32_t* __restrict__ counts) {
  __shared__ int c[MOE_MAX_E];
  for (int e = threadIdx.x; e < MOE_MAX_E; e += MOE_CHUNK) c[e] = 0;
  __syncthreads();
  const int t = blockIdx.x * MOE_CHUNK + threadIdx.x;
  if (t < T)
    for (int j = 0; j < k; ++j) {
      const int e = idx[(size_t)t * k + j];
      if (e >= 0 && e < E) atomicAdd(&c[e], 1);           // integer count: order does not matter
    }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += MOE_CHUNK) counts[(size_t)blockIdx.x * E + e] = c[e];
}

// one workgroup: per expert the exclusive prefix over the token chunks, the padded segment
// offsets, and the row block -> expert table (-1 past the last segment)
__global__ __launch_bounds__(256) void moe_offsets_kernel(const int32_t* __restrict__ counts, int nblk, int E,
                                                          int32_t* __restrict__ base,
                                                          int32_t* __restrict__ expert_rows,
                                                          int32_t* __restrict__ tile_group, int n_tiles) {
  __shared__ int total[MOE_MAX_E];
  __shared__ int rows[MOE_MAX_E + 1];
  for (int e = threadIdx.x; e < E; e += 256) {
    int run = 0;
    for (int b = 0; b < nblk; ++b) {
      base[(size_t)b * E + e] = run;
      run += counts[(size_t)b * E + e];
    }
    total[e] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int off = 0;
    for (int e = 0; e < E; ++e) {
      rows[e] = off;
      off += (total[e] + MOE_PAD - 1) / MOE_PAD * MOE_PAD;
    }
    rows[E] = off;
  }
  __syncthreads();
  for (int e = threadIdx.x; e <= E; e += 256) expert_rows[e] = rows[e];
  for (int tile = threadIdx.x; tile < n_tiles; tile += 256) {
    const int r = tile * MOE_PAD;
    int g = -1;
    for (int e = 0; e < E; ++e)
      if (r >= rows[e] && r < rows[e + 1]) g = e;
    tile_group[tile] = g;
  }
}

__global__ void moe_fill_i32_kernel(int32_t* __restrict__ p, int32_t v, long n) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// slot of every (token, choice): segment offset + tokens of earlier chunks + rank inside the
// chunk (token order); also the inverse tables row -> token and row -> gate
__global__ __launch_bounds__(MOE_CHUNK) void moe_slot_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ gate, int T, int E, int k,
    const int32_t* __restrict__ base, const int32_t* __restrict__ expert_rows,
    int32_t* __restrict__ slot, int32_t* __restrict__ row_token, float* __restrict__ row_gate, int cap) {
  __shared__ int wcnt[MOE_CHUNK / 64][MOE_MAX_E];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * MOE_CHUNK + threadIdx.x;
  int mine[MOE_MAX_K], rank[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    mine[j] = (t < T && j < k) ? idx[(size_t)t * k + j] : -1;
    rank[j] = 0;
  }
  const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int e = 0; e < E; ++e) {
    bool has = false;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) has = has || mine[j] == e;
    const unsigned long long b = __ballot(has);
    const int before = __popcll(b & below);
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (mine[j] == e) rank[j] = before;
    if (lane == 0) wcnt[wave][e] = __popcll(b);
  }
  __syncthreads();
  if (t >= T) return;
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    const int e = mine[j];
    if (j >= k || e < 0 || e >= E) continue;
    int r = rank[j];
    for (int w = 0; w < wave; ++w) r += wcnt[w][e];
    const int s = expert_rows[e] + base[(size_t)blockIdx.x * E + e] + r;
    slot[(size_t)t * k + j] = s;
    if (s >= 0 && s < cap) {
      row_token[s] = t;
      row_gate[s] = gate[(size_t)t * k + j];
    }
  }
}

// ---- row movement ------------------------------------------------------------------------------
// dst[row] = scale(row) * src[row_token[row]]  (zeros for padding rows); scale = row_gate or 1
template <typename T>
__global__ void moe_gather_kernel(const T* __restrict__ src, const int32_t* __restrict__ row_token,
                                  const float* __restrict__ row_gate, T* __restrict__ dst, int rows,
                                  int d, int n_src) {
  constexpr int VEC = Elt<T>::VEC;
  const int per = d / VEC;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)rows * per) return;
  const int row = (int)(gid / per), c = (int)(gid % per) * VEC;
  const int t = row_token[row];
  float v[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] = 0.f;
  if (t >= 0 && t < n_src) {
    load16(src + (size_t)t * d + c, v);
    if (row_gate) {
      const float g = row_gate[row];
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] *= g;
    }
  }
  store16(dst + (size_t)row * d + c, v);
}

// out[t] = (res ? res[t] : 0) + sum_j w(t,j) * rows[slot[t,j]],  w = gate or 1; choices in order
template <typename T>
__global__ void moe_combine_kernel(const T* __restrict__ rows, const int32_t* __restrict__ slot,
                                   const float* __restrict__ gate, const T* __restrict__ res,
                                   T* __restrict__ out, int Tn, int k, int d, int cap) {
  constexpr int VEC = Elt<T>::VEC;
  const int per = d / VEC;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)Tn * per) return;
  const int t = (int)(gid / per), c = (int)(gid % per) * VEC;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  for (int j = 0; j < k; ++j) {
    const int s = slot[(size_t)t * k + j];
    if (s < 0 || s >= cap) continue;
    float v[VEC];
    load16(rows + (size_t)s * d + c, v);
    const float g = gate ? gate[(size_t)t * k + j] : 1.0f;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = fmaf(g, v[e], acc[e]);
  }
  if (res) {
    float r[VEC];
    load16(res + (size_t)t * d + c, r);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += r[e];
  }
  store16(out + (size_t)t * d + c, acc);
}

// ---- router backward (one wavefront per token) ------------------------------------------------
// dgate[t,j] = <dm[t], y_rows[slot[t,j]]>; then through the gate normalisation and the
// softmax: dlogit_e = p_e (dp_e - sum_e' p_e' dp_e'), dp nonzero on the chosen experts only
template <typename T>
__global__ __launch_bounds__(256) void moe_router_bwd_kernel(
    const T* __restrict__ dm, const T* __restrict__ y_rows, const int32_t* __restrict__ slot,
    const int32_t* __restrict__ idx, const float* __restrict__ gate, const float* __restrict__ probs,
    T* __restrict__ dlogits, int Tn, int E, int k, int d, int cap) {
  constexpr int VEC = Elt<T>::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= Tn) return;
  float dg[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    dg[j] = 0.f;
    if (j >= k) continue;
    const int s = slot[(size_t)t * k + j];
    if (s < 0 || s >= cap) continue;
    float part = 0.f;
    for (int c = lane * VEC; c < d; c += WAVE * VEC) {
      float a[VEC], b[VEC];
      load16(dm + (size_t)t * d + c, a);
      load16(y_rows + (size_t)s * d + c, b);
#pragma unroll
      for (int e = 0; e < VEC; ++e) part = fmaf(a[e], b[e], part);
    }
    dg[j] = wave_sum(part);
  }
  float ssum = 0.f, dot_g = 0.f;
  int who[MOE_MAX_K];
  float ps[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    who[j] = -1; ps[j] = 0.f;
    if (j >= k) continue;
    who[j] = idx[(size_t)t * k + j];
    ps[j] = probs[(size_t)t * E + who[j]];
    ssum += ps[j];
    dot_g += dg[j] * gate[(size_t)t * k + j];
  }
  float dsel[MOE_MAX_K], dot_p = 0.f;
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    dsel[j] = j < k ? (dg[j] - dot_g) / ssum : 0.f;
    dot_p += ps[j] * dsel[j];
  }
  for (int e = lane; e < E; e += WAVE) {
    float dp = 0.f;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (who[j] == e) dp = dsel[j];
    dlogits[(size_t)t * E + e] = Elt<T>::from_f(probs[(size_t)t * E + e] * (dp - dot_p));
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
int moe_row_capacity(int T, int E, int k) {
  const long r = (long)T * k + (long)E * (MOE_PAD - 1);
  return (int)((r + MOE_PAD - 1) / MOE_PAD * MOE_PAD);
}

size_t moe_layout_scratch_bytes(int T, int E) {
  const size_t nblk = (size_t)cdiv(T, MOE_CHUNK);
  return 2 * align_up(nblk * E * sizeof(int32_t), 256);      // counts + base
}

bm_status moe_check(int E, int k, int d, int dtype) {
  if (E < 1 || E > MOE_MAX_E) { set_error("moe: %d experts outside [1,%d]", E, MOE_MAX_E); return BM_ERR_UNSUPPORTED; }
  if (k < 1 || k > MOE_MAX_K || k > E) { set_error("moe: top_k %d outside [1,min(%d,E)]", k, MOE_MAX_K); return BM_ERR_UNSUPPORTED; }
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (d % vec) { set_error("moe: hidden %d not a multiple of %d", d, vec); return BM_ERR_UNSUPPORTED; }
  return BM_OK;
}

bm_status moe_route(const float* logits, int T, int E, int k, float* probs, int32_t* idx, float* gate,
                    hipStream_t st) {
  hipLaunchKernelGGL(moe_route_kernel, dim3(cdiv(T, 4)), dim3(256), 0, st, logits, T, E, k, probs, idx, gate);
  BM_CHECK_LAUNCH("moe_route");
  return BM_OK;
}

bm_status moe_layout(const MoeTables& m, int T, int E, int k, void* scratch, hipStream_t st) {
  const int nblk = cdiv(T, MOE_CHUNK);
  int32_t* counts = (int32_t*)scratch;
  int32_t* base = (int32_t*)((char*)scratch + align_up((size_t)nblk * E * sizeof(int32_t), 256));
  hipLaunchKernelGGL(moe_count_kernel, dim3(nblk), dim3(MOE_CHUNK), 0, st, m.idx, T, E, k, counts);
  hipLaunchKernelGGL(moe_offsets_kernel, dim3(1), dim3(256), 0, st, counts, nblk, E, base, m.expert_rows,
                     m.tile_group, m.cap / MOE_PAD);
  hipLaunchKernelGGL(moe_fill_i32_kernel, dim3(cdiv(m.cap, 256)), dim3(256), 0, st, m.row_token, -1, (long)m.cap);
  hipLaunchKernelGGL(moe_slot_kernel, dim3(nblk), dim3(MOE_CHUNK), 0, st, m.idx, m.gate, T, E, k, base,
                     m.expert_rows, m.slot, m.row_token, m.row_gate, m.cap);
  BM_CHECK_LAUNCH("moe_layout");
  return BM_OK;
}

bm_status moe_gather(int dtype, const void* src, const MoeTables& m, int use_gate, void* dst, int d, int T,
                     hipStream_t st) {
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  const long n = (long)m.cap * (d / vec);
  const float* rg = use_gate ? m.row_gate : nullptr;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(moe_gather_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const bf16_t*)src,
                       m.row_token, rg, (bf16_t*)dst, m.cap, d, T);
  else
    hipLaunchKernelGGL(moe_gather_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const float*)src,
                       m.row_token, rg, (float*)dst, m.cap, d, T);
  BM_CHECK_LAUNCH("moe_gather");
  return BM_OK;
}

bm_status moe_combine(int dtype, const void* rows, const MoeTables& m, int use_gate, const void* res,
                      void* out, int T, int k, int d, hipStream_t st) {
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  const long n = (long)T * (d / vec);
  const float* g = use_gate ? m.gate : nullptr;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(moe_combine_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const bf16_t*)rows,
                       m.slot, g, (const bf16_t*)res, (bf16_t*)out, T, k, d, m.cap);
  else
    hipLaunchKernelGGL(moe_combine_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const float*)rows,
                       m.slot, g, (const float*)res, (float*)out, T, k, d, m.cap);
  BM_CHECK_LAUNCH("moe_combine");
  return BM_OK;
}

bm_status moe_router_backward(int dtype, const void* dm, const void* y_rows, const MoeTables& m,
                              void* dlogits, int T, int E, int k, int d, hipStream_t st) {
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(moe_router_bwd_kernel<bf16_t>, dim3(cdiv(T, 4)), dim3(256), 0, st, (const bf16_t*)dm,
                       (const bf16_t*)y_rows, m.slot, m.idx, m.gate, m.probs, (bf16_t*)dlogits, T, E, k, d, m.cap);
  else
    hipLaunchKernelGGL(moe_router_bwd_kernel<float>, dim3(cdiv(T, 4)), dim3(256), 0, st, (const float*)dm,
                       (const float*)y_rows, m.slot, m.idx, m.gate, m.probs, (float*)dlogits, T, E, k, d, m.cap);
  BM_CHECK_LAUNCH("moe_router_backward");
  return BM_OK;
}

}  // namespace bm
