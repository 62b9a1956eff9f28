// bf16 MFMA GEMM (placeholder: nothing is routed here yet).
#include "common.h"

namespace bm {

bool gemm_mfma_supported(int, int, int, int, int, int, int, int, const GemmEpilogue&) { return false; }
size_t gemm_mfma_scratch_bytes(int, int, int, int) { return 0; }
bm_status gemm_mfma(int, int, int, int, const void*, int, const void*, int, void*, int,
                    const GemmEpilogue&, void*, size_t, hipStream_t) {
  set_error("gemm_mfma: not built"); return BM_ERR_UNSUPPORTED;
}

}  // namespace bm
