/* Two-stream (text / image) adaLN transformer block with joint attention: forward and
 * backward on one GPU.
 *
 * The paper names its generator as a multimodal diffusion transformer built from attention
 * operators (Sec. 4.1) and gives no arithmetic; the reading built here is the two-stream block
 * of that literature.  Every sample has a text token sequence and an image token sequence.
 * Per stream s, with its OWN parameters:
 *   mod_s = silu(c) W_ada_s^T + b_ada_s = [shift1, scale1, gate1, shift2, scale2, gate2]
 *   h     = LN0(x_s) (1 + scale1) + shift1                 (LN0: LayerNorm without affine)
 *   q,k,v = h W_qkv_s^T + b_qkv_s ;  with qk_norm: q <- q / rms_dh(q) * gq_s, k likewise
 *   o     = softmax attention, bidirectional, over [text tokens ; image tokens] of the sample
 *   x1    = x_s + gate1 (o W_o_s^T + b_o_s)
 *   y_s   = x1 + gate2 (gelu(LN0(x1)(1 + scale2) + shift2) W_up_s^T + b_up_s) W_down_s^T + b_down_s)
 * c is one conditioning row per sample, shared by both streams.
 *
 * Layout: each stream is packed on its own, x_s [T_s, hidden] row-major with cu_s[S+1] the
 * per-sample offsets (a sample needs at least one token in each stream).  All buffers are the
 * caller's; weight gradients are fp32 and ACCUMULATE (+=), dcond is overwritten.  Work is
 * enqueued on the given stream without host synchronisation; errors are return codes with a
 * message in bm_last_error(), and an invalid call launches nothing.
 */
#ifndef BIGMAC_MMDIT_H
#define BIGMAC_MMDIT_H

#include "bigmac_block.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  bm_block_desc block;   /* hidden, n_q_heads = n_kv_heads, head_dim, mlp_hidden, norm_eps, dtype;
                            norm must be BM_NORM_ADALN, act GELU, mask bidirectional, rope 0,
                            linear_bias 1, n_experts 0                                          */
  int32_t qk_norm;       /* 0/1: RMS normalisation of q and k over head_dim with per-stream gains */
  float   qk_norm_eps;
} bm_mmdit_desc;

typedef struct {
  bm_block_params stream[2];    /* [0] text, [1] image: w/b_qkv, w/b_o, w/b_up, w/b_down, w/b_ada  */
  void* q_norm_g[2];            /* [head_dim] per stream (qk_norm only)                            */
  void* k_norm_g[2];
} bm_mmdit_params;              /* gradients: same layout, fp32                                    */

/* Size limit of every call: (T_text + T_img) x widest row (the larger of the packed q|k|v
 * width, mlp_hidden and hidden) must stay below 2^31 elements; larger packs return
 * BM_ERR_INVALID_ARG. */
bm_status bm_mmdit_sizes(const bm_mmdit_desc* desc, int32_t T_text, int32_t T_img, int32_t S,
                         size_t* saved_bytes, size_t* scratch_bytes);

bm_status bm_mmdit_forward(const bm_mmdit_desc* desc, const bm_mmdit_params* w,
                           const void* x_text, const void* x_img,
                           const int32_t* cu_text_dev, const int32_t* cu_text_host,
                           const int32_t* cu_img_dev, const int32_t* cu_img_host, int32_t S,
                           const void* cond /* [S, hidden] */, void* y_text, void* y_img,
                           void* saved, void* scratch, size_t scratch_bytes, void* hip_stream);

bm_status bm_mmdit_backward(const bm_mmdit_desc* desc, const bm_mmdit_params* w,
                            const void* x_text, const void* x_img,
                            const void* dy_text, const void* dy_img,
                            const int32_t* cu_text_dev, const int32_t* cu_text_host,
                            const int32_t* cu_img_dev, const int32_t* cu_img_host, int32_t S,
                            const void* cond, const void* saved, void* dx_text, void* dx_img,
                            const bm_mmdit_params* grads, void* dcond,
                            void* scratch, size_t scratch_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
