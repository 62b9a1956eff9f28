// bf16 MFMA flash attention (placeholder: nothing is routed here yet).
#include "common.h"

namespace bm {

bool attention_mfma_supported(const AttnArgs&) { return false; }
bm_status attention_forward_mfma(const AttnArgs&, void*, float*, hipStream_t) {
  set_error("attention_forward_mfma: not built"); return BM_ERR_UNSUPPORTED;
}
size_t attention_backward_mfma_scratch_bytes(int, int, int, int) { return 0; }
bm_status attention_backward_mfma(const AttnArgs&, const void*, const void*, const float*, void*,
                                  void*, void*, int, void*, size_t, hipStream_t) {
  set_error("attention_backward_mfma: not built"); return BM_ERR_UNSUPPORTED;
}

}  // namespace bm
