// One rank's share of context-parallel attention: chunk-pair forward / backward on the packed
// variable-length attention kernels (queries and keys/values packed separately), the merge of
// partial outputs by their log-sum-exp, and the fp32 sum of gradient parts.
#include "common.h"
#include "../../include/bigmac_cp_attention.h"

namespace bm {

namespace {

struct MergeParts {
  const void* o[BM_CP_MAX_PARTS];
  const float* lse[BM_CP_MAX_PARTS];
  int n;
};

// one thread: 16 bytes of one (row, head).  Weights exp(lse_c - max) are taken relative to the
// largest part, so the largest weight is exactly 1 and nothing overflows.
template <typename T>
__global__ void cp_merge_kernel(MergeParts p, T* __restrict__ o, float* __restrict__ lse, int Tq, int Hq, int dh) {
  constexpr int VEC = Elt<T>::VEC;
  const int per = dh / VEC;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)Tq * Hq * per) return;
  const int c = (int)(gid % per) * VEC;
  const int h = (int)((gid / per) % Hq);
  const int t = (int)(gid / ((long)per * Hq));
  float m = -INFINITY;
  for (int i = 0; i < p.n; ++i) m = fmaxf(m, p.lse[i][(size_t)h * Tq + t]);
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  float z = 0.f;
  if (m > -INFINITY) {
    for (int i = 0; i < p.n; ++i) {
      const float w = expf(p.lse[i][(size_t)h * Tq + t] - m);      // exp(-inf) = 0 for an empty part
      if (w == 0.f) continue;
      float v[VEC];
      load16((const T*)p.o[i] + ((size_t)t * Hq + h) * dh + c, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = fmaf(w, v[e], acc[e]);
      z += w;
    }
    const float inv = 1.0f / z;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] *= inv;
  }
  store16(o + ((size_t)t * Hq + h) * dh + c, acc);
  if (c == 0) lse[(size_t)h * Tq + t] = m > -INFINITY ? m + logf(z) : -INFINITY;
}

struct SumParts {
  const void* p[BM_CP_MAX_PARTS];
  int n;
};

template <typename T>
__global__ void cp_sum_parts_kernel(SumParts p, T* __restrict__ out, long n) {
  constexpr int VEC = Elt<T>::VEC;
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (i >= n) return;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  for (int c = 0; c < p.n; ++c) {
    float v[VEC];
    load16((const T*)p.p[c] + i, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += v[e];
  }
  store16(out + i, acc);
}

bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// validity of both packings; fills the chunk fields of `a`
bm_status check_chunks(int dtype, int mask, int Hq, int Hkv, int dh, int ld_q, int ld_kv,
                       const int32_t* cu_q_dev, const int32_t* cu_q_host, const int32_t* cu_k_dev,
                       const int32_t* cu_k_host, int S, AttnArgs* a) {
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "cp attention: dtype %d", dtype);
  BM_ARG_CHECK(mask == BM_MASK_BIDIRECTIONAL || mask == BM_MASK_CAUSAL, "cp attention: mask %d", mask);
  BM_ARG_CHECK(Hq > 0 && Hkv > 0 && Hq % Hkv == 0, "cp attention: heads %d/%d", Hq, Hkv);
  switch (dh) {
    case 8: case 16: case 32: case 64: case 72: case 128: break;
    default: set_error("cp attention: head_dim %d unsupported (8,16,32,64,72,128)", dh); return BM_ERR_UNSUPPORTED;
  }
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(ld_q >= Hq * dh && ld_q % vec == 0, "cp attention: query row stride %d", ld_q);
  BM_ARG_CHECK(ld_kv >= Hkv * dh && ld_kv % vec == 0, "cp attention: key/value row stride %d", ld_kv);
  BM_ARG_CHECK(S >= 1 && cu_q_dev && cu_q_host && cu_k_dev && cu_k_host, "cp attention: S = %d or NULL offsets", S);
  BM_ARG_CHECK(cu_q_host[0] == 0 && cu_k_host[0] == 0, "cp attention: offsets must start at 0");
  int max_q = 0, max_k = 0;
  for (int s = 0; s < S; ++s) {
    const int lq = cu_q_host[s + 1] - cu_q_host[s], lk = cu_k_host[s + 1] - cu_k_host[s];
    BM_ARG_CHECK(lq >= 0 && lk >= 0, "cp attention: sequence %d has a negative length", s);
    BM_ARG_CHECK(mask != BM_MASK_CAUSAL || lq == lk,
                 "cp attention: a causal pair is a chunk with itself, sequence %d has %d queries and %d keys", s, lq, lk);
    max_q = lq > max_q ? lq : max_q;
    max_k = lk > max_k ? lk : max_k;
  }
  a->dtype = dtype; a->causal = mask == BM_MASK_CAUSAL; a->Hq = Hq; a->Hkv = Hkv; a->dh = dh;
  a->ld_qkv = ld_q; a->cu_dev = cu_q_dev; a->cu_host = cu_q_host; a->S = S; a->T = cu_q_host[S];
  a->max_seqlen = max_q;
  a->cu_k_dev = cu_k_dev; a->cu_k_host = cu_k_host; a->Tk = cu_k_host[S]; a->ld_kv = ld_kv; a->max_klen = max_k;
  return BM_OK;
}

}  // namespace

}  // namespace bm

using namespace bm;

extern "C" bm_status bm_cp_attention_forward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                                             const void* q, int32_t ld_q, const void* k, const void* v,
                                             int32_t ld_kv, const int32_t* cu_q_dev, const int32_t* cu_q_host,
                                             const int32_t* cu_k_dev, const int32_t* cu_k_host, int32_t S,
                                             void* o_part, float* lse_part, void* hip_stream) {
  AttnArgs a{};
  BM_RETURN_IF(check_chunks(dtype, mask, Hq, Hkv, dh, ld_q, ld_kv, cu_q_dev, cu_q_host, cu_k_dev, cu_k_host, S, &a));
  if (a.T == 0) return BM_OK;
  BM_ARG_CHECK(q && o_part && lse_part && al16(q) && al16(o_part), "cp attention: NULL or misaligned query-side tensor");
  BM_ARG_CHECK(a.Tk == 0 || (k && v && al16(k) && al16(v)), "cp attention: NULL or misaligned key/value tensor");
  a.q = q; a.k = k; a.v = v;
  return attention_forward(a, o_part, lse_part, (hipStream_t)hip_stream);
}

extern "C" bm_status bm_cp_attention_merge(int32_t dtype, int32_t Hq, int32_t dh, int32_t Tq, int32_t n_parts,
                                           const void* const* o_parts, const float* const* lse_parts, void* o,
                                           float* lse, void* hip_stream) {
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "cp merge: dtype %d", dtype);
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(Hq > 0 && dh > 0 && dh % vec == 0 && Tq >= 0, "cp merge: bad sizes Hq=%d dh=%d Tq=%d", Hq, dh, Tq);
  BM_ARG_CHECK(n_parts >= 1 && n_parts <= BM_CP_MAX_PARTS, "cp merge: %d parts (1..%d)", n_parts, BM_CP_MAX_PARTS);
  BM_ARG_CHECK(o_parts && lse_parts && o && lse && al16(o), "cp merge: NULL or misaligned tensor");
  MergeParts p{};
  p.n = n_parts;
  for (int i = 0; i < n_parts; ++i) {
    BM_ARG_CHECK(o_parts[i] && lse_parts[i] && al16(o_parts[i]), "cp merge: part %d is NULL or misaligned", i);
    BM_ARG_CHECK(o_parts[i] != o, "cp merge: o aliases part %d", i);
    p.o[i] = o_parts[i]; p.lse[i] = lse_parts[i];
  }
  if (Tq == 0) return BM_OK;
  const long n = (long)Tq * Hq * (dh / vec);
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope prof(PROF_ELEMENTWISE, (double)(n_parts + 1) * Tq * Hq * dh * (double)elt_size(dtype), st);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(cp_merge_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, p, (bf16_t*)o, lse, Tq, Hq, dh);
  else
    hipLaunchKernelGGL(cp_merge_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, p, (float*)o, lse, Tq, Hq, dh);
  BM_CHECK_LAUNCH("cp_merge");
  return BM_OK;
}

extern "C" size_t bm_cp_attention_backward_scratch_bytes(int32_t Hq, int32_t Hkv, int32_t dh, int32_t Tq,
                                                         int32_t Tk) {
  if (Hq <= 0 || Hkv <= 0 || dh <= 0 || Tq < 0 || Tk < 0) return 0;
  return attention_backward_scratch_bytes(Hq, Hkv, dh, Tq > 0 ? Tq : 1, Tk > 0 ? Tk : 1);
}

extern "C" bm_status bm_cp_attention_backward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                                              const void* q, int32_t ld_q, const void* k, const void* v,
                                              int32_t ld_kv, const void* o, const void* d_o, const float* lse,
                                              const int32_t* cu_q_dev, const int32_t* cu_q_host,
                                              const int32_t* cu_k_dev, const int32_t* cu_k_host, int32_t S,
                                              void* dq_part, int32_t ld_dq, void* dk_part, void* dv_part,
                                              int32_t ld_dkv, void* scratch, size_t scratch_bytes,
                                              void* hip_stream) {
  AttnArgs a{};
  BM_RETURN_IF(check_chunks(dtype, mask, Hq, Hkv, dh, ld_q, ld_kv, cu_q_dev, cu_q_host, cu_k_dev, cu_k_host, S, &a));
  if (a.T == 0 && a.Tk == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(ld_dq >= Hq * dh && ld_dq % vec == 0, "cp attention backward: dq row stride %d", ld_dq);
  BM_ARG_CHECK(ld_dkv >= Hkv * dh && ld_dkv % vec == 0, "cp attention backward: dk/dv row stride %d", ld_dkv);
  BM_ARG_CHECK(a.T == 0 || (q && o && d_o && lse && dq_part && al16(q) && al16(o) && al16(d_o) && al16(dq_part)),
               "cp attention backward: NULL or misaligned query-side tensor");
  BM_ARG_CHECK(a.Tk == 0 || (k && v && dk_part && dv_part && al16(k) && al16(v) && al16(dk_part) && al16(dv_part)),
               "cp attention backward: NULL or misaligned key/value-side tensor");
  const size_t need = bm_cp_attention_backward_scratch_bytes(Hq, Hkv, dh, a.T, a.Tk);
  if (need > scratch_bytes || !scratch) {
    set_error("cp attention backward needs %zu scratch bytes, got %zu", need, scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  a.q = q; a.k = k; a.v = v; a.ld_dkv = ld_dkv;
  return attention_backward(a, o, d_o, lse, dq_part, dk_part, dv_part, ld_dq, scratch, scratch_bytes,
                            (hipStream_t)hip_stream);
}

extern "C" bm_status bm_cp_sum_parts(int32_t dtype, int64_t n, int32_t n_parts, const void* const* parts,
                                     void* out, void* hip_stream) {
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "cp sum: dtype %d", dtype);
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(n >= 0 && n % vec == 0, "cp sum: length %lld is not a multiple of %d", (long long)n, vec);
  BM_ARG_CHECK(n_parts >= 1 && n_parts <= BM_CP_MAX_PARTS, "cp sum: %d parts (1..%d)", n_parts, BM_CP_MAX_PARTS);
  BM_ARG_CHECK(parts && out && al16(out), "cp sum: NULL or misaligned tensor");
  SumParts p{};
  p.n = n_parts;
  for (int i = 0; i < n_parts; ++i) {
    BM_ARG_CHECK(parts[i] && al16(parts[i]), "cp sum: part %d is NULL or misaligned", i);
    p.p[i] = parts[i];
  }
  if (n == 0) return BM_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope prof(PROF_ELEMENTWISE, (double)(n_parts + 1) * n * (double)elt_size(dtype), st);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(cp_sum_parts_kernel<bf16_t>, dim3(cdiv(n / vec, 256)), dim3(256), 0, st, p, (bf16_t*)out, (long)n);
  else
    hipLaunchKernelGGL(cp_sum_parts_kernel<float>, dim3(cdiv(n / vec, 256)), dim3(256), 0, st, p, (float*)out, (long)n);
  BM_CHECK_LAUNCH("cp_sum_parts");
  return BM_OK;
}
