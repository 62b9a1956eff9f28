// Variable-length attention with plain fp32 arithmetic: one thread owns one
// query row (forward, dq) or one key row (dk, dv), key/query tiles are staged
// in LDS and read as broadcasts.  It serves the fp32 check path and head sizes
// the MFMA kernels do not take.  No atomics: each output element has one owner.
//
//   forward : o = softmax(q k^T / sqrt(dh) + mask) v,  lse = log sum exp (scaled scores)
//   backward: p = exp(s - lse), dv = p^T do, dp = do v^T, ds = p * (dp - delta),
//             dq = ds k / sqrt(dh), dk = ds^T q / sqrt(dh), delta = rowsum(do * o)
#include "common.h"

namespace bm {

namespace {

constexpr int BQ = 128;   // rows per workgroup (one per thread)
constexpr int BT = 32;    // rows of the streamed tile

template <typename T, int DH, bool CAUSAL>
__global__ __launch_bounds__(BQ) void attn_fwd_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, int ld, int ldk,
    const int32_t* __restrict__ cu, const int32_t* __restrict__ cuk, T* __restrict__ o, int ldo,
    float* __restrict__ lse, int Ttot, int group, float scale) {
  __shared__ float Ks[BT][DH];
  __shared__ float Vs[BT][DH];
  const int s = blockIdx.y, hq = blockIdx.z, hk = hq / group;
  const int lo = cu[s], L = cu[s + 1] - lo;
  const int lok = cuk[s], Lk = cuk[s + 1] - lok;     // keys/values may be packed on their own
  const int q0 = blockIdx.x * BQ;
  if (q0 >= L) return;
  const int qi = q0 + threadIdx.x;
  const bool active = qi < L;
  float qr[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = active ? Elt<T>::to_f(q[(size_t)(lo + qi) * ld + hq * DH + c]) * scale : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int kend = CAUSAL ? min(Lk, q0 + BQ) : Lk;
  for (int k0 = 0; k0 < kend; k0 += BT) {
    for (int idx = threadIdx.x; idx < BT * DH; idx += BQ) {
      int r = idx / DH, c = idx % DH, kj = k0 + r;
      bool ok = kj < Lk;
      Ks[r][c] = ok ? Elt<T>::to_f(k[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
      Vs[r][c] = ok ? Elt<T>::to_f(v[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
    }
    __syncthreads();
    if (active) {
      float sc[BT];
      float tmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < BT; ++j) {
        int kj = k0 + j;
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < DH; ++c) d = fmaf(qr[c], Ks[j][c], d);
        bool ok = kj < Lk && (!CAUSAL || kj <= qi);
        sc[j] = ok ? d : -INFINITY;
        tmax = fmaxf(tmax, sc[j]);
      }
      if (tmax > -INFINITY) {
        float mn = fmaxf(m, tmax);
        float corr = expf(m - mn);
        l *= corr;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] *= corr;
#pragma unroll
        for (int j = 0; j < BT; ++j) {
          float p = expf(sc[j] - mn);   // exp(-inf) = 0 for masked keys
          l += p;
#pragma unroll
          for (int c = 0; c < DH; ++c) acc[c] = fmaf(p, Vs[j][c], acc[c]);
        }
        m = mn;
      }
    }
    __syncthreads();
  }
  if (active) {
    float inv = l > 0.f ? 1.0f / l : 0.f;       // no visible key in this chunk: o = 0, lse = -inf
#pragma unroll
    for (int c = 0; c < DH; ++c)
      o[(size_t)(lo + qi) * ldo + hq * DH + c] = Elt<T>::from_f(acc[c] * inv);
    lse[(size_t)hq * Ttot + lo + qi] = l > 0.f ? m + logf(l) : -INFINITY;
  }
}

template <typename T, int DH>
__global__ void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ d_o, int ldo,
                                  float* __restrict__ delta, int Ttot, int Hq) {
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)Ttot * Hq) return;
  int t = (int)(gid / Hq), hq = (int)(gid % Hq);
  const T* po = o + (size_t)t * ldo + hq * DH;
  const T* pd = d_o + (size_t)t * ldo + hq * DH;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < DH; ++c) s = fmaf(Elt<T>::to_f(po[c]), Elt<T>::to_f(pd[c]), s);
  delta[(size_t)hq * Ttot + t] = s;
}

template <typename T, int DH, bool CAUSAL>
__global__ __launch_bounds__(BQ) void attn_dq_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, int ld, int ldk,
    const T* __restrict__ d_o, int ldo, const float* __restrict__ lse,
    const float* __restrict__ delta, const int32_t* __restrict__ cu, const int32_t* __restrict__ cuk,
    T* __restrict__ dq, int ldd, int Ttot, int group, float scale) {
  __shared__ float Ks[BT][DH];
  __shared__ float Vs[BT][DH];
  const int s = blockIdx.y, hq = blockIdx.z, hk = hq / group;
  const int lo = cu[s], L = cu[s + 1] - lo;
  const int lok = cuk[s], Lk = cuk[s + 1] - lok;
  const int q0 = blockIdx.x * BQ;
  if (q0 >= L) return;
  const int qi = q0 + threadIdx.x;
  const bool active = qi < L;
  float qr[DH], dor[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = active ? Elt<T>::to_f(q[(size_t)(lo + qi) * ld + hq * DH + c]) * scale : 0.f;
    dor[c] = active ? Elt<T>::to_f(d_o[(size_t)(lo + qi) * ldo + hq * DH + c]) : 0.f;
    acc[c] = 0.f;
  }
  const float my_lse = active ? lse[(size_t)hq * Ttot + lo + qi] : 0.f;
  const float my_delta = active ? delta[(size_t)hq * Ttot + lo + qi] : 0.f;
  const int kend = CAUSAL ? min(Lk, q0 + BQ) : Lk;
  for (int k0 = 0; k0 < kend; k0 += BT) {
    for (int idx = threadIdx.x; idx < BT * DH; idx += BQ) {
      int r = idx / DH, c = idx % DH, kj = k0 + r;
      bool ok = kj < Lk;
      Ks[r][c] = ok ? Elt<T>::to_f(k[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
      Vs[r][c] = ok ? Elt<T>::to_f(v[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
    }
    __syncthreads();
    if (active) {
      for (int j = 0; j < BT; ++j) {
        int kj = k0 + j;
        if (kj >= Lk || (CAUSAL && kj > qi)) break;
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < DH; ++c) {
          sc = fmaf(qr[c], Ks[j][c], sc);
          dp = fmaf(dor[c], Vs[j][c], dp);
        }
        float ds = expf(sc - my_lse) * (dp - my_delta);
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] = fmaf(ds, Ks[j][c], acc[c]);
      }
    }
    __syncthreads();
  }
  if (active) {
#pragma unroll
    for (int c = 0; c < DH; ++c)
      dq[(size_t)(lo + qi) * ldd + hq * DH + c] = Elt<T>::from_f(acc[c] * scale);
  }
}

// One thread per key row of one kv head; the q heads of the group and the query
// tiles are walked in a fixed order, so dk/dv sums are reproducible.
template <typename T, int DH, bool CAUSAL>
__global__ __launch_bounds__(BQ) void attn_dkdv_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, int ld, int ldk,
    const T* __restrict__ d_o, int ldo, const float* __restrict__ lse,
    const float* __restrict__ delta, const int32_t* __restrict__ cuq, const int32_t* __restrict__ cuk,
    T* __restrict__ dk, T* __restrict__ dv, int ldd, int Ttot, int group, float scale) {
  // this thread's key row lives in the key/value packing (cuk, ldk); queries, dO, lse and
  // delta (Ttot rows per head) in the queries' packing (cuq, ld)
  __shared__ float Qs[BT][DH];
  __shared__ float Ds[BT][DH];
  __shared__ float Ls[BT], Dl[BT];
  const int s = blockIdx.y, hk = blockIdx.z;
  const int lok = cuk[s], Lk = cuk[s + 1] - lok;
  const int lo = cuq[s], L = cuq[s + 1] - lo;
  const int kb = blockIdx.x * BQ;
  if (kb >= Lk) return;
  const int kj = kb + threadIdx.x;
  const bool active = kj < Lk;
  float kr[DH], vr[DH], dkr[DH], dvr[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    kr[c] = active ? Elt<T>::to_f(k[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
    vr[c] = active ? Elt<T>::to_f(v[(size_t)(lok + kj) * ldk + hk * DH + c]) : 0.f;
    dkr[c] = 0.f; dvr[c] = 0.f;
  }
  const int qstart = CAUSAL ? (kb / BT) * BT : 0;
  for (int g = 0; g < group; ++g) {
    const int hq = hk * group + g;
    for (int q0 = qstart; q0 < L; q0 += BT) {
      for (int idx = threadIdx.x; idx < BT * DH; idx += BQ) {
        int r = idx / DH, c = idx % DH, qi = q0 + r;
        bool ok = qi < L;
        Qs[r][c] = ok ? Elt<T>::to_f(q[(size_t)(lo + qi) * ld + hq * DH + c]) * scale : 0.f;
        Ds[r][c] = ok ? Elt<T>::to_f(d_o[(size_t)(lo + qi) * ldo + hq * DH + c]) : 0.f;
      }
      if (threadIdx.x < BT) {
        int qi = q0 + threadIdx.x;
        bool ok = qi < L;
        Ls[threadIdx.x] = ok ? lse[(size_t)hq * Ttot + lo + qi] : 0.f;
        Dl[threadIdx.x] = ok ? delta[(size_t)hq * Ttot + lo + qi] : 0.f;
      }
      __syncthreads();
      if (active) {
        for (int i = 0; i < BT; ++i) {
          int qi = q0 + i;
          if (qi >= L) break;
          if (CAUSAL && kj > qi) continue;
          float sc = 0.f, dp = 0.f;
#pragma unroll
          for (int c = 0; c < DH; ++c) {
            sc = fmaf(Qs[i][c], kr[c], sc);
            dp = fmaf(Ds[i][c], vr[c], dp);
          }
          float p = expf(sc - Ls[i]);
          float ds = p * (dp - Dl[i]);
#pragma unroll
          for (int c = 0; c < DH; ++c) {
            dvr[c] = fmaf(p, Ds[i][c], dvr[c]);
            dkr[c] = fmaf(ds, Qs[i][c], dkr[c]);   // Qs already carries 1/sqrt(dh)
          }
        }
      }
      __syncthreads();
    }
  }
  if (active) {
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      dk[(size_t)(lok + kj) * ldd + hk * DH + c] = Elt<T>::from_f(dkr[c]);
      dv[(size_t)(lok + kj) * ldd + hk * DH + c] = Elt<T>::from_f(dvr[c]);
    }
  }
}

template <typename T, int DH, bool CAUSAL>
bm_status fwd_launch(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
  dim3 grid(cdiv(a.max_seqlen, BQ), a.S, a.Hq);
  hipLaunchKernelGGL((attn_fwd_generic_kernel<T, DH, CAUSAL>), grid, dim3(BQ), 0, st, (const T*)a.q,
                     (const T*)a.k, (const T*)a.v, a.ld_qkv, a.kv_ld(), a.cu_dev, a.kv_cu_dev(), (T*)o,
                     a.Hq * a.dh, lse, a.T, a.Hq / a.Hkv, 1.0f / sqrtf((float)a.dh));
  BM_CHECK_LAUNCH("attn_fwd_generic");
  return BM_OK;
}

template <typename T, int DH, bool CAUSAL>
bm_status bwd_launch(const AttnArgs& a, const void* o, const void* d_o, const float* lse, void* dq,
                     void* dk, void* dv, int ldd, float* delta, hipStream_t st) {
  const int ldo = a.Hq * a.dh;
  const float scale = 1.0f / sqrtf((float)a.dh);
  long n = (long)a.T * a.Hq;
  if (n > 0) {
    hipLaunchKernelGGL((attn_delta_kernel<T, DH>), dim3(cdiv(n, 256)), dim3(256), 0, st, (const T*)o,
                       (const T*)d_o, ldo, delta, a.T, a.Hq);
    hipLaunchKernelGGL((attn_dq_generic_kernel<T, DH, CAUSAL>), dim3(cdiv(a.max_seqlen, BQ), a.S, a.Hq),
                       dim3(BQ), 0, st, (const T*)a.q, (const T*)a.k, (const T*)a.v, a.ld_qkv, a.kv_ld(),
                       (const T*)d_o, ldo, lse, delta, a.cu_dev, a.kv_cu_dev(), (T*)dq, ldd, a.T,
                       a.Hq / a.Hkv, scale);
  }
  if (a.kv_T() > 0)
    hipLaunchKernelGGL((attn_dkdv_generic_kernel<T, DH, CAUSAL>),
                       dim3(cdiv(a.kv_max_len(), BQ), a.S, a.Hkv), dim3(BQ), 0, st, (const T*)a.q,
                       (const T*)a.k, (const T*)a.v, a.ld_qkv, a.kv_ld(), (const T*)d_o, ldo, lse, delta,
                       a.cu_dev, a.kv_cu_dev(), (T*)dk, (T*)dv, a.ld_dkv ? a.ld_dkv : ldd, a.T,
                       a.Hq / a.Hkv, scale);
  BM_CHECK_LAUNCH("attn_bwd_generic");
  return BM_OK;
}

#define BM_DH_SWITCH(CALL)                      \
  switch (a.dh) {                               \
    case 8: CALL(8); break;                     \
    case 16: CALL(16); break;                   \
    case 32: CALL(32); break;                   \
    case 64: CALL(64); break;                   \
    case 72: CALL(72); break;                   \
    case 128: CALL(128); break;                 \
    default:                                    \
      set_error("attention: head_dim %d unsupported (8,16,32,64,72,128)", a.dh); \
      return BM_ERR_UNSUPPORTED;                \
  }

}  // namespace

bm_status attention_forward_generic(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
  if (a.T == 0) return BM_OK;
#define BM_CALL(D)                                                                             \
  if (a.dtype == BM_DTYPE_BF16)                                                                \
    return a.causal ? fwd_launch<bf16_t, D, true>(a, o, lse, st) : fwd_launch<bf16_t, D, false>(a, o, lse, st); \
  else                                                                                         \
    return a.causal ? fwd_launch<float, D, true>(a, o, lse, st) : fwd_launch<float, D, false>(a, o, lse, st)
  BM_DH_SWITCH(BM_CALL)
#undef BM_CALL
  return BM_OK;
}

bm_status attention_backward_generic(const AttnArgs& a, const void* o, const void* d_o,
                                     const float* lse, void* dq, void* dk, void* dv, int ldd,
                                     float* delta, hipStream_t st) {
  if (a.T == 0 && a.kv_T() == 0) return BM_OK;
#define BM_CALL(D)                                                                             \
  if (a.dtype == BM_DTYPE_BF16)                                                                \
    return a.causal ? bwd_launch<bf16_t, D, true>(a, o, d_o, lse, dq, dk, dv, ldd, delta, st)  \
                    : bwd_launch<bf16_t, D, false>(a, o, d_o, lse, dq, dk, dv, ldd, delta, st); \
  else                                                                                         \
    return a.causal ? bwd_launch<float, D, true>(a, o, d_o, lse, dq, dk, dv, ldd, delta, st)   \
                    : bwd_launch<float, D, false>(a, o, d_o, lse, dq, dk, dv, ldd, delta, st)
  BM_DH_SWITCH(BM_CALL)
#undef BM_CALL
  return BM_OK;
}

}  // namespace bm
