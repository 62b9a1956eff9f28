/* One rank's share of context-parallel attention (Sec. 3.3 "Context parallelism"): the tokens of
 * every sequence are partitioned over the ranks of a context-parallel group; a rank keeps the
 * queries of its chunk and is handed the keys/values of the chunks one after the other (the
 * ring-attention scheme the paper cites).  These entry points are what ONE rank computes on
 * its GPU; moving the chunks between GPUs is not part of this library.
 *
 * For one (query chunk, key/value chunk) pair, per query row i and head:
 *     s_ij = <q_i, k_j> / sqrt(head_dim) over the visible keys j of that chunk,
 *     lse_i = log sum_j exp(s_ij)  (-inf without a visible key),  o_i = sum_j exp(s_ij - lse_i) v_j  (0 then).
 * Partial results of several chunks merge to attention over all their keys:
 *     lse_i = log sum_c exp(lse_i^c),   o_i = sum_c exp(lse_i^c - lse_i) o_i^c .
 * Backward of one pair takes the MERGED o, lse of the query rows and dO and yields that pair's
 * dq (to be summed over key/value chunks) and dk, dv (to be summed over query chunks).
 *
 * Layout: queries [Tq, ld_q] and keys/values [Tk, ld_kv] are packed per chunk with their own
 * per-sequence offsets cu_q[S+1], cu_k[S+1] over the same S sequences; a sequence may have no
 * row in a chunk.  mask = BM_MASK_CAUSAL means "the key/value chunk IS the query chunk" (key
 * position <= query position; cu_q must equal cu_k); a chunk that lies wholly before the
 * query chunk is passed with BM_MASK_BIDIRECTIONAL, one that lies after it is not passed.
 * o / dO / dq rows are n_q_heads*head_dim wide unless a stride is given; lse is [n_q_heads, Tq]
 * fp32.  All buffers are the caller's, device memory unless marked host; work is enqueued on the
 * stream without host synchronisation; results are bit-reproducible (no atomics).  Errors are
 * return codes with a message in bm_last_error(); an invalid call launches nothing.
 */
#ifndef BIGMAC_CP_ATTENTION_H
#define BIGMAC_CP_ATTENTION_H

#include "bigmac_block.h"

#ifdef __cplusplus
extern "C" {
#endif

#define BM_CP_MAX_PARTS 16

bm_status bm_cp_attention_forward(int32_t dtype, int32_t mask, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim, const void* q, int32_t ld_q, const void* k,
                                  const void* v, int32_t ld_kv, const int32_t* cu_q_dev,
                                  const int32_t* cu_q_host, const int32_t* cu_k_dev,
                                  const int32_t* cu_k_host, int32_t S, void* o_part, float* lse_part,
                                  void* hip_stream);

/* o, lse <- merge of n_parts (<= BM_CP_MAX_PARTS) partial results; o_parts / lse_parts are HOST
 * arrays of device pointers; a part whose lse is -inf contributes nothing; o may alias none of
 * the parts. */
bm_status bm_cp_attention_merge(int32_t dtype, int32_t n_q_heads, int32_t head_dim, int32_t Tq,
                                int32_t n_parts, const void* const* o_parts,
                                const float* const* lse_parts, void* o, float* lse, void* hip_stream);

size_t bm_cp_attention_backward_scratch_bytes(int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                              int32_t Tq, int32_t Tk);

/* dq_part [Tq, ld_dq], dk_part / dv_part [Tk, ld_dkv] are overwritten (rows of sequences that are
 * empty on the other side become zero). */
bm_status bm_cp_attention_backward(int32_t dtype, int32_t mask, int32_t n_q_heads, int32_t n_kv_heads,
                                   int32_t head_dim, const void* q, int32_t ld_q, const void* k,
                                   const void* v, int32_t ld_kv, const void* o, const void* d_o,
                                   const float* lse, const int32_t* cu_q_dev, const int32_t* cu_q_host,
                                   const int32_t* cu_k_dev, const int32_t* cu_k_host, int32_t S,
                                   void* dq_part, int32_t ld_dq, void* dk_part, void* dv_part,
                                   int32_t ld_dkv, void* scratch, size_t scratch_bytes, void* hip_stream);

/* out[i] = sum over the parts of parts[c][i], i < n, added in fp32 in part order and rounded once
 * (the sum of a rank's dq parts, or of the dk / dv parts that travelled round the ring). */
bm_status bm_cp_sum_parts(int32_t dtype, int64_t n, int32_t n_parts, const void* const* parts, void* out,
                          void* hip_stream);

/* ---- encoder -> LLM layout conversion (Sec. 3.3: encoder and LLM may use different context-parallel
 * degrees; the handoff then re-lays the modality embeddings with an all-to-all, and the encoder unit
 * grows to pp_size * llm_cp / enc_cp microbatches).  Host-side planning only.
 *
 * Layout rule on both sides: a sequence of length L is cut into C contiguous position ranges, chunk c
 * = positions [c*L/C, (c+1)*L/C) (integer division); a rank's buffer holds its chunk of every
 * sequence, sequence by sequence.  Encoder sequences are the images (image_lens[n_images] patch
 * tokens each), LLM sequences the documents (cu_docs[n_docs+1], offsets into the packed microbatch);
 * image_rows[k] is the row of that pack which encoder token k fills, tokens counted image by image
 * (distinct rows).  All pointers are host memory.
 *
 * Output: counts[e*llm_cp + l] = tokens that encoder rank e sends to LLM rank l; src_rows / dst_rows
 * [sum of image_lens]: for each pair (e, l) in that order, the rows of rank e's buffer to send, ascending,
 * and the rows of rank l's buffer where they land. */
bm_status bm_cp_conversion_plan(int32_t enc_cp, int32_t llm_cp, int32_t n_images, const int32_t* image_lens,
                                const int32_t* image_rows, int32_t n_docs, const int32_t* cu_docs,
                                int32_t* counts, int32_t* src_rows, int32_t* dst_rows);

/* *unit_size = pp_size * llm_cp / enc_cp (Sec. 3.3); an error unless the division is exact. */
bm_status bm_cp_encoder_unit_size(int32_t pp_size, int32_t llm_cp, int32_t enc_cp, int32_t* unit_size);

/* Row moves that apply a plan (or any handoff index list, Sec. 3.2 "Module handoff") on device
 * memory: dst[i, :] = src[rows[i], :] and dst[rows[i], :] = src[i, :] for i < n; rows is a device
 * array of distinct indices, width in elements (a multiple of 16 bytes). */
bm_status bm_row_gather(int32_t dtype, const void* src, const int32_t* rows_dev, void* dst, int32_t n,
                        int32_t width, void* hip_stream);
bm_status bm_row_scatter(int32_t dtype, const void* src, const int32_t* rows_dev, void* dst, int32_t n,
                         int32_t width, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
