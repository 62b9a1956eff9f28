/*
 * bigmac_block.h -- C-ABI of the MI355X (gfx950) library that runs the forward
 * and backward pass of one packed, variable-length transformer block, plus the
 * host-side nested schedule and the single-GPU micro-unit executor built on it.
 *
 * Background.  The paper's training pipeline (Sec. 3) nests modality-encoder
 * and generator units into an unchanged LLM pipeline schedule; the work every
 * unit executes is the forward/backward of transformer blocks (ViT encoder
 * blocks, LLM decoder blocks, diffusion-transformer generator blocks; Sec. 2.1
 * "Multimodal LLMs", "Model heterogeneity") over packed sequences (Sec. 3.3).
 * The paper gives no arithmetic for the blocks; each is the standard pre-norm
 * residual block of its kind:
 *
 *   h   = N1(x)                       LayerNorm | RMSNorm | LN0 + adaLN modulate
 *   qkv = h Wqkv^T (+ bqkv)           rows of Wqkv: all q heads, all k heads, all v heads
 *   q,k = RoPE(q,k)                   rotate-half pairs (i, i+dh/2), angle p*base^(-2i/dh),
 *                                     p = position inside the token's own sequence
 *   o   = softmax(q k^T/sqrt(dh) + mask) v     per sequence and head; q head a uses
 *                                     kv head a / (Hq/Hkv); mask causal or none
 *   x1  = x + [gate1 *] (o Wo^T (+ bo))
 *   h2  = N2(x1)
 *   m   = gelu_erf(h2 W1^T + b1) W2^T + b2   |   (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T
 *   y   = x1 + [gate2 *] m
 *
 *   adaLN: [shift1,scale1,gate1,shift2,scale2,gate2] = split6(silu(cond_s) Wada^T + bada)
 *          per sequence s, N(x) = LN0(x) * (1 + scale) + shift.
 *
 * Conventions for every entry point
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  The caller owns every buffer; the library never allocates or
 *     frees device memory and keeps no pointer after a call returns (an
 *     executor object keeps the pointers it was created with).
 *   - Tensors are row-major, token-major ([T, features]); bf16 storage with
 *     fp32 accumulation (dtype 0) or fp32 storage (dtype 1, the check path).
 *     Device pointers must be 16-byte aligned.
 *   - Work is enqueued on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream); no call synchronises with the host.
 *   - Errors are return codes; bm_last_error() gives the text of the last
 *     failure on the calling thread.  Nothing aborts or throws.
 */
#ifndef BIGMAC_BLOCK_H
#define BIGMAC_BLOCK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BM_OK = 0,
  BM_ERR_INVALID_ARG = -1,          /* NULL/misaligned pointer, bad cu_seqlens, bad sizes   */
  BM_ERR_UNSUPPORTED = -2,          /* a shape or variant the kernels do not cover          */
  BM_ERR_WORKSPACE_TOO_SMALL = -3,  /* scratch_bytes below what bm_block_sizes reports      */
  BM_ERR_HIP = -4                   /* a HIP runtime call failed (text in bm_last_error)    */
} bm_status;

enum { BM_NORM_LAYERNORM = 0, BM_NORM_RMSNORM = 1, BM_NORM_ADALN = 2 };
enum { BM_ACT_GELU = 0, BM_ACT_SWIGLU = 1 };
enum { BM_MASK_BIDIRECTIONAL = 0, BM_MASK_CAUSAL = 1 };
enum { BM_DTYPE_BF16 = 0, BM_DTYPE_FP32 = 1 };

/* Shape and variant of one block. hidden must equal n_q_heads*head_dim. */
typedef struct {
  int32_t hidden, n_q_heads, n_kv_heads, head_dim, mlp_hidden;
  int32_t norm;         /* BM_NORM_*                                                       */
  int32_t act;          /* BM_ACT_GELU: two-matrix MLP;  BM_ACT_SWIGLU: w_up is [2F,d],
                           gate rows first, then linear rows                               */
  int32_t mask;         /* BM_MASK_*; attention is always block-diagonal by cu_seqlens     */
  int32_t rope;         /* 0/1                                                             */
  float   rope_base;
  float   norm_eps;
  int32_t linear_bias;  /* 0/1: biases on the four linear layers                           */
  int32_t dtype;        /* BM_DTYPE_*                                                      */
  int32_t deterministic;/* ignored: every kernel here is free of floating-point atomics, so
                           results are run-to-run bit-identical whatever this field holds  */
  int32_t n_experts;    /* 0: dense FFN.  > 0 (<= 256): mixture-of-experts FFN (the paper's
                           LLM backbone, Sec. 4.1): router logits h W_r^T, softmax over the
                           experts, the top_k most probable experts (ties: lower index) with
                           their probabilities renormalised to sum 1 as gates, every expert a
                           SwiGLU FFN of width mlp_hidden, no token dropped.  Needs
                           act = SwiGLU, linear_bias = 0, a norm other than adaLN.            */
  int32_t top_k;        /* 1..min(8, n_experts)                                             */
} bm_block_desc;

/* Parameters (storage dtype) -- and, with the same field meaning, their
 * gradients (always fp32).  Weight matrices are [out, in] row-major.  Fields a
 * variant does not own must be NULL. */
typedef struct {
  void *norm1_g, *norm1_b;   /* [d]             (LayerNorm: g,b; RMSNorm: g)               */
  void *w_qkv,  *b_qkv;      /* [(Hq+2Hkv)dh,d], [(Hq+2Hkv)dh]                             */
  void *w_o,    *b_o;        /* [d, Hq*dh], [d]                                            */
  void *norm2_g, *norm2_b;
  void *w_up,   *b_up;       /* [F,d] or [2F,d];  [F] or [2F]; with experts [E,2F,d]       */
  void *w_down, *b_down;     /* [d,F], [d]; with experts [E,d,F]                           */
  void *w_ada,  *b_ada;      /* [6d,d], [6d]    (adaLN only)                               */
  void *w_router;            /* [E,d]           (mixture of experts only)                  */
} bm_block_params;

/* Last error text of the calling thread ("" if none). Never NULL. */
const char* bm_last_error(void);

/* Bytes the caller must provide for `saved` (kept from forward to backward)
 * and for `scratch` (free after each call; max over forward and backward).
 * T packed tokens in S sequences, none longer than max_seqlen.
 * Size limit of every block call: rows x widest row (the larger of the packed
 * q|k|v width, the up-projection width and hidden; rows = T, or the padded
 * expert capacity of a mixture block) must stay below 2^31 elements; larger
 * packs return BM_ERR_INVALID_ARG and are to be split by the caller. */
bm_status bm_block_sizes(const bm_block_desc* desc, int32_t T, int32_t S, int32_t max_seqlen,
                         size_t* saved_bytes, size_t* scratch_bytes);

/* Forward of one block.
 *   w               parameters (dev pointers inside a host struct)
 *   x      dev      [T, hidden]   block input (the caller keeps it for backward)
 *   cu_seqlens_dev  [S+1] int32   sequence boundaries, cu[0]=0, cu[S]=T, increasing
 *   cu_seqlens_host [S+1] int32   the same values in host memory (validated, and used
 *                                 to build launch grids without a device round trip)
 *   cond   dev      [S, hidden]   per-sequence conditioning (adaLN), else NULL
 *   y      dev      [T, hidden]   output; must not alias x, saved or scratch
 *   saved  dev      saved_bytes   written here, read by bm_block_backward
 *   scratch dev     scratch_bytes
 * Returns BM_ERR_INVALID_ARG for bad arguments (nothing is launched then). */
bm_status bm_block_forward(const bm_block_desc* desc, const bm_block_params* w,
                           const void* x, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, int32_t S, int32_t T,
                           int32_t max_seqlen, const void* cond, void* y, void* saved,
                           void* scratch, size_t scratch_bytes, void* hip_stream);

/* Where a mixture-of-experts forward left its routing decisions: device pointers INTO `saved`
 * (valid as long as the caller keeps that buffer; nothing is copied or launched).
 *   expert_out  -> int32 [T, top_k]  experts chosen for each token, most probable first
 *   gate_out    -> fp32  [T, top_k]  their gates (probabilities renormalised to sum 1)
 * T and S are those of the forward call.  The choice is an integer taken from floating-point
 * router logits (Sec. 4.1 names the mixture-of-experts backbone, Sec. 3.3 its load imbalance),
 * so a caller that compares two implementations, or balances load, reads it here.
 * BM_ERR_INVALID_ARG for a block without experts. */
bm_status bm_block_moe_routing(const bm_block_desc* desc, int32_t T, int32_t S, const void* saved,
                               const int32_t** expert_out /* host */, const float** gate_out /* host */);

/* Backward of one block.
 *   x, cond, cu_*   as given to the forward call that filled `saved`
 *   dy     dev      [T, hidden]  upstream gradient
 *   dx     dev      [T, hidden]  gradient w.r.t. x (overwritten)
 *   grads           fp32 buffers shaped like the parameters; the call ADDS its
 *                   contribution (the caller zeroes them once per optimiser step:
 *                   the accumulation semantics of Sec. 3.2 "Module handoff")
 *   dcond  dev      [S, hidden] storage dtype, overwritten (adaLN), else NULL */
bm_status bm_block_backward(const bm_block_desc* desc, const bm_block_params* w,
                            const void* x, const void* dy, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, int32_t S, int32_t T,
                            int32_t max_seqlen, const void* cond, const void* saved,
                            void* dx, const bm_block_params* grads, void* dcond,
                            void* scratch, size_t scratch_bytes, void* hip_stream);

/* ---- single operations of the path (same kernels the block calls use) ------------- */

/* C = op(A) op(B) (+bias) with fp32 accumulation; layouts
 *   0 "NT": C[M,N]  = A[M,K] B[N,K]^T        (linear forward,  Y = X W^T)
 *   1 "NN": C[M,N]  = A[M,K] B[K,N]          (input gradient,  dX = dY W)
 *   2 "TN": C[M,N] += A[K,M]^T B[K,N]        (weight gradient, dW += dY^T X; C is fp32)
 * A, B (and C for layouts 0/1, bias[N]) are in the storage dtype; leading dimensions
 * in elements.  scratch may be NULL when scratch_bytes is 0; bm_gemm_scratch_bytes
 * gives what the split reduction of layout 2 wants. */
size_t    bm_gemm_scratch_bytes(int32_t layout, int32_t M, int32_t N, int32_t K, int32_t dtype);
bm_status bm_gemm(int32_t layout, int32_t dtype, int32_t M, int32_t N, int32_t K,
                  const void* A, int32_t lda, const void* B, int32_t ldb,
                  void* C, int32_t ldc, const void* bias,
                  void* scratch, size_t scratch_bytes, void* hip_stream);

/* Variable-length attention, q:[T,Hq,dh] k,v:[T,Hkv,dh] rows of one packed qkv
 * buffer with row stride ld_qkv elements; o:[T,Hq*dh]; lse:[Hq,T] fp32 (natural-log
 * sum-exp of the scaled scores of each row).  Softmax scale 1/sqrt(dh). */
bm_status bm_attention_forward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                               const void* q, const void* k, const void* v, int32_t ld_qkv,
                               const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                               int32_t S, int32_t T, int32_t max_seqlen,
                               void* o, float* lse, void* hip_stream);

/* Gradients dq,dk,dv (rows of one packed buffer with row stride ld_dqkv, fully
 * overwritten) from do:[T,Hq*dh], the forward's q,k,v,o and lse.
 * scratch: bm_attention_backward_scratch_bytes(...) bytes. */
size_t    bm_attention_backward_scratch_bytes(int32_t Hq, int32_t Hkv, int32_t dh, int32_t T);
bm_status bm_attention_backward(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                                const void* q, const void* k, const void* v, int32_t ld_qkv,
                                const void* o, const void* d_o, const float* lse,
                                const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                                int32_t S, int32_t T, int32_t max_seqlen,
                                void* dq, void* dk, void* dv, int32_t ld_dqkv,
                                void* scratch, size_t scratch_bytes, void* hip_stream);

/* The same operation for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is
 * bm_attention_backward with the workspace taken from a fixed array of
 * BM_ATTENTION_STATIC_SCRATCH_BYTES that is part of the library's device code (each GPU the
 * library runs on holds its own copy until the process ends); the call allocates and frees
 * nothing.  Arguments, outputs and validation are those of bm_attention_backward.  Shapes whose
 * workspace (bm_attention_backward_scratch_bytes) exceeds the array return
 * BM_ERR_WORKSPACE_TOO_SMALL and launch nothing.  Every call on a GPU shares that GPU's array:
 * calls that overlap on one GPU (two streams, two threads) race on it and must be serialised
 * by the caller.  The array keeps the previous call's contents; nothing in it needs clearing,
 * because every byte the kernels read from it is written earlier in the same call.
 * bm_attention_backward_static_capacity() returns BM_ATTENTION_STATIC_SCRATCH_BYTES. */
#define BM_ATTENTION_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
size_t    bm_attention_backward_static_capacity(void);
bm_status bm_attention_backward_static(int32_t dtype, int32_t mask, int32_t Hq, int32_t Hkv, int32_t dh,
                                       const void* q, const void* k, const void* v, int32_t ld_qkv,
                                       const void* o, const void* d_o, const float* lse,
                                       const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                                       int32_t S, int32_t T, int32_t max_seqlen,
                                       void* dq, void* dk, void* dv, int32_t ld_dqkv, void* hip_stream);

/* ---- measurement: per-kernel-class timing ------------------------------------------- */

/* Between bm_profile_begin() and bm_profile_end() every kernel group the library
 * launches is bracketed by a pair of HIP events recorded on the launch stream.
 * bm_profile_end synchronises with those events and returns, per class, the
 * summed elapsed milliseconds, the summed algorithmic work (flops for GEMM and
 * attention classes, bytes for the HBM-bound classes) and the number of launches.
 * Outputs are host arrays of BM_PROF_CLASSES entries.  Not thread safe; measuring
 * tool only (it serialises neighbouring kernels at the event boundaries). */
enum { BM_PROF_GEMM_NT = 0, BM_PROF_GEMM_NN = 1, BM_PROF_GEMM_TN = 2, BM_PROF_ATTN_FWD = 3,
       BM_PROF_ATTN_BWD = 4, BM_PROF_NORM = 5, BM_PROF_ELEMENTWISE = 6, BM_PROF_CLASSES = 7 };
bm_status bm_profile_begin(void);
bm_status bm_profile_end(double* ms /* host */, double* work /* host */, int64_t* launches /* host */);

/* Yardsticks for the roofline denominators (the caller times them on the stream):
 * bm_probe_mfma launches `blocks` workgroups of 4 wavefronts that each issue iters*16
 * register-resident v_mfma_f32_32x32x16_bf16 (32768 flop each) with no memory traffic;
 * bm_probe_copy streams bytes (multiple of 16) from src to dst (dev), 2*bytes of HBM traffic. */
bm_status bm_probe_mfma(int32_t blocks, int32_t iters, float* out_dev, void* hip_stream);
bm_status bm_probe_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream);
/* bm_probe_mfma with a choice of instruction shape (shape16 = 0: 32x32x16, 16 MFMAs per iteration;
 * 1: 16x16x32, 64 per iteration: iters * 2^19 or iters * 2^20 flop per wavefront) and of operand
 * data (random_operands = 0: zeros; 1: pseudo-random values of unit scale).  The clock the chip
 * holds under matrix load depends on the operand data, so the rate on random operands is the
 * ceiling that applies to real activations.  Other values of the two switches: BM_ERR_INVALID_ARG. */
bm_status bm_probe_mfma_ex(int32_t blocks, int32_t iters, int32_t shape16, int32_t random_operands,
                           float* out_dev, void* hip_stream);
/* The two legs of the copy on their own: bm_probe_read streams bytes (multiple of 16) from
 * src_dev and writes nothing (out_dev: 256 words of dev memory that keep the loads alive), with
 * `blocks` workgroups of 256 threads each holding `unroll` (1, 4 or 8) 16-byte loads in flight;
 * bm_probe_fill writes bytes to dst_dev with `blocks` workgroups. */
bm_status bm_probe_read(const void* src_dev, size_t bytes, int32_t blocks, int32_t unroll,
                        void* out_dev, void* hip_stream);
bm_status bm_probe_fill(void* dst_dev, size_t bytes, int32_t blocks, void* hip_stream);
/* LDS yardstick (measurement contract, like the probes above).  512 workgroups of 4 wavefronts,
 * two per CU; per wavefront and iteration, `what` -- a sum of 1: 16 KiB of row-fragment reads
 * (ds_read_b128), 2: 16 KiB of transposed-fragment reads (ds_read_b64_tr_b16), 4: 8 KiB of LDS
 * stores (ds_write_b128), 8: 8 KiB of 16-byte loads that write LDS directly -- moves through the
 * LDS.  Supported: 1, 2, 4, 8, 5 and 9 (reads next to either kind of fill, the ratio of a GEMM
 * slice).  src_dev (dev, at least 512 KiB) is read by the direct loads only and may be NULL
 * otherwise; out_dev: one word (dev), never written.  The caller times the launch.
 * bm_probe_issue: 256 workgroups of 4 wavefronts, iters x 4 groups of one 32x32x16 MFMA followed
 * by n_valu (0, 4 or 8) independent vector instructions: what a group takes beyond the MFMA's
 * 32 clocks is vector issue time that found no room beside it.
 * Both return BM_ERR_INVALID_ARG for any other `what` / n_valu, before anything is launched. */
bm_status bm_probe_lds(int32_t what, int32_t iters, const void* src_dev, size_t src_bytes, void* out_dev,
                       void* hip_stream);
bm_status bm_probe_issue(int32_t n_valu, int32_t iters, float* out_dev, void* hip_stream);

/* ---- nested schedule (host only; Sec. 3.1 and the BuildSchedule figure) ------------ */

enum { BM_OP_ENC_FWD = 0, BM_OP_ENC_BWD = 1, BM_OP_LLM_FWD = 2, BM_OP_LLM_BWD = 3,
       BM_OP_GEN_FWD = 4, BM_OP_GEN_BWD = 5 };
enum { BM_ORDER_NESTED = 0,             /* the paper's nested order                         */
       BM_ORDER_COMPUTE_EFFICIENT = 1,  /* all encoder forwards first, backwards last       */
       BM_ORDER_SEQUENTIAL = 2 };       /* one unit at a time                               */

/* Writes the op stream for M microbatches in units of unit_size, W warm-up
 * encoder units, an LLM 1F1B order with llm_depth units in flight.  Each op is
 * two int32: (opcode, index) where index is a unit id for ENC and GEN ops and
 * a microbatch id for LLM ops.  n_ops: in = capacity of ops_out in ops,
 * out = ops written (or needed, with BM_ERR_INVALID_ARG, if capacity is short). */
bm_status bm_build_schedule(int32_t order, int32_t M, int32_t unit_size, int32_t W,
                            int32_t llm_depth, int32_t has_generator,
                            int32_t* ops_out /* host */, int32_t* n_ops /* host */);

/* Checks an op stream for dependency safety (encoder output before its LLM
 * forwards, generator between the unit's last forward and first backward,
 * encoder backward after the unit's last LLM backward, each op exactly once)
 * and reports the peak number of live encoder/generator units and LLM
 * microbatches.  peak_out: host int32[3] or NULL. */
bm_status bm_check_schedule(const int32_t* ops /* host */, int32_t n_ops, int32_t M,
                            int32_t unit_size, int32_t has_generator, int32_t* peak_out);

/* ---- single-GPU micro-unit executor (Sec. 3.2: opcode interpreter, runtime buffers,
 *      module handoff; local part only, no communication operators) --------------------
 *
 * One pipeline stage's share on one GPU: M LLM microbatches through n_llm_blocks decoder
 * blocks, with encoder units (n_enc_blocks ViT blocks over the images of unit_size
 * microbatches) and generator units (n_gen_blocks adaLN blocks, one sequence of
 * gen_tokens_per_image latent tokens per image) nested between them by an op stream from
 * bm_build_schedule.  Glue (stand-in structure, the paper only says "projectors"):
 *   feat   = enc_out proj_in^T                  [enc tokens, llm.hidden]
 *   llm_in = base, with row image_rows[i] replaced by feat row i     (embed_preprocess)
 *   cond   = llm_out[image_last_row] proj_out^T [images, gen.hidden]
 *   loss_u = 0.5 * mean((gen_out - targets)^2)  per unit (written to loss[u]);
 *   without generator: loss_m = <llm_out, out_grad> per microbatch (written to loss[m]).
 * Activations live in fixed slots carved from the caller's arena (enc_slots encoder
 * units, llm_slots LLM microbatches, one generator unit); an op that finds no free slot
 * fails with BM_ERR_WORKSPACE_TOO_SMALL.  Weight gradients accumulate (+=) as in
 * bm_block_backward.  All structs are host memory; pointers inside are device pointers
 * unless named *_host. */
typedef struct bm_executor bm_executor;

typedef struct {
  bm_block_desc enc, llm, gen;                 /* same dtype; gen.norm must be BM_NORM_ADALN     */
  int32_t n_enc_blocks, n_llm_blocks, n_gen_blocks;   /* n_gen_blocks = 0: no generator          */
  int32_t M, unit_size;
  int32_t gen_tokens_per_image;
} bm_executor_config;

typedef struct {
  const bm_block_params *enc, *llm, *gen;     /* host arrays [n_*_blocks]                        */
  void *proj_in;                              /* [llm.hidden, enc.hidden]                        */
  void *proj_out;                             /* [gen.hidden, llm.hidden] (with generator)       */
} bm_executor_params;                         /* gradients: same layout, fp32                    */

typedef struct {                              /* one LLM microbatch                              */
  int32_t T, S;
  const int32_t *cu_dev, *cu_host;            /* [S+1] documents                                 */
  const void* base;                           /* [T, llm.hidden] text-token activations          */
  int32_t n_image_rows;
  const int32_t* image_rows;                  /* [n_image_rows] LLM row of each encoder token of
                                                 this microbatch, in the unit's encoder order    */
  int32_t n_images;
  const int32_t* image_last_row;              /* [n_images] LLM row conditioning each image      */
  const void* out_grad;                       /* [T, llm.hidden], used without generator         */
} bm_microbatch;

typedef struct {                              /* one unit: the images of its microbatches, in
                                                 microbatch order                                */
  int32_t T, S;                               /* encoder tokens and images                       */
  const int32_t *cu_dev, *cu_host;            /* [S+1] one sequence per image                    */
  const void* patches;                        /* [T, enc.hidden] encoder input                   */
  const int32_t *gen_cu_dev, *gen_cu_host;    /* [S+1] = k * gen_tokens_per_image (generator)    */
  const void* latents;                        /* [S*gen_tokens_per_image, gen.hidden]            */
  const void* targets;                        /* same shape                                      */
} bm_unit;

/* Arena bytes needed for the given slot counts (sized for the largest unit/microbatch). */
bm_status bm_executor_arena_bytes(const bm_executor_config* cfg, const bm_microbatch* mbs,
                                  const bm_unit* units, int32_t enc_slots, int32_t llm_slots,
                                  size_t* bytes);
/* The executor keeps every pointer it is given (they must outlive it); arena is dev memory. */
bm_status bm_executor_create(const bm_executor_config* cfg, const bm_executor_params* w,
                             const bm_executor_params* grads, const bm_microbatch* mbs /* [M] */,
                             const bm_unit* units /* [ceil(M/unit_size)] */, void* arena,
                             size_t arena_bytes, int32_t enc_slots, int32_t llm_slots,
                             bm_executor** out);
/* ops: (opcode, index) pairs as written by bm_build_schedule; checked with bm_check_schedule. */
bm_status bm_executor_load_schedule(bm_executor* ex, const int32_t* ops, int32_t n_ops);
/* Runs the loaded op stream once on the stream. loss: dev float[M], overwritten per unit or
 * microbatch as described above.  No host synchronisation. */
bm_status bm_executor_execute(bm_executor* ex, float* loss, void* hip_stream);
/* The same run with a HIP event recorded on the stream around every op; synchronises with the
 * last event and fills op_ms (host double[n_ops]: milliseconds of each op of the loaded stream)
 * and, when not NULL, live_bytes (host double[n_ops]: live activation bytes after each op).
 * A measuring tool: it feeds measured operator times to bm_pipeline_replay (Sec. 3.1). */
bm_status bm_executor_execute_timed(bm_executor* ex, float* loss, double* op_ms /* host */,
                                    double* live_bytes /* host or NULL */, void* hip_stream);
/* High-water mark, over the last execute, of the bytes of saved activations and
 * inter-module feature/gradient buffers that were alive at the same time (weights,
 * gradients and scratch excluded), and its encoder-unit part. */
size_t bm_executor_peak_activation_bytes(const bm_executor* ex);
size_t bm_executor_peak_encoder_bytes(const bm_executor* ex);
void   bm_executor_destroy(bm_executor* ex);

#ifdef __cplusplus
}
#endif
#endif /* BIGMAC_BLOCK_H */
