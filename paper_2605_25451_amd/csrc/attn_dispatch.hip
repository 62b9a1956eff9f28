// Attention back-end selection: MFMA flash kernels for bf16 with head sizes
// they cover, the generic fp32-arithmetic kernels otherwise.
#include "common.h"

namespace bm {

bool attention_mfma_supported(const AttnArgs& a);
bm_status attention_forward_mfma(const AttnArgs& a, void* o, float* lse, hipStream_t st);
size_t attention_backward_mfma_scratch_bytes(int Hq, int Hkv, int dh, int Tq, int Tk);
bm_status attention_backward_mfma(const AttnArgs& a, const void* o, const void* d_o, const float* lse,
                                  void* dq, void* dk, void* dv, int ld_dqkv, void* scratch,
                                  size_t scratch_bytes, hipStream_t st);

// unmasked (query, key) pairs inside the sequences
static double attn_pairs(const AttnArgs& a) {
  double pairs = 0;
  const int32_t* ck = a.kv_cu_host();
  for (int s = 0; s < a.S; ++s) {
    double L = a.cu_host[s + 1] - a.cu_host[s], Lk = ck[s + 1] - ck[s];
    pairs += a.causal ? L * (L + 1) / 2 : L * Lk;
  }
  return pairs;
}

bm_status attention_forward(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
  ProfScope prof(PROF_ATTN_FWD, 4.0 * a.dh * a.Hq * attn_pairs(a), st);
  if (attention_mfma_supported(a)) return attention_forward_mfma(a, o, lse, st);
  return attention_forward_generic(a, o, lse, st);
}

size_t attention_backward_scratch_bytes(int Hq, int Hkv, int dh, int Tq, int Tk) {
  size_t generic = align_up((size_t)Hq * Tq * sizeof(float), 256);   // delta
  size_t mfma = attention_backward_mfma_scratch_bytes(Hq, Hkv, dh, Tq, Tk);
  return generic > mfma ? generic : mfma;
}

size_t attention_backward_scratch_bytes(int Hq, int Hkv, int dh, int T) {
  return attention_backward_scratch_bytes(Hq, Hkv, dh, T, T);
}

bm_status attention_backward(const AttnArgs& a, const void* o, const void* d_o, const float* lse,
                             void* dq, void* dk, void* dv, int ld_dqkv, void* scratch,
                             size_t scratch_bytes, hipStream_t st) {
  ProfScope prof(PROF_ATTN_BWD, 10.0 * a.dh * a.Hq * attn_pairs(a), st);
  if (attention_mfma_supported(a))
    return attention_backward_mfma(a, o, d_o, lse, dq, dk, dv, ld_dqkv, scratch, scratch_bytes, st);
  return attention_backward_generic(a, o, d_o, lse, dq, dk, dv, ld_dqkv, (float*)scratch, st);
}

}  // namespace bm
