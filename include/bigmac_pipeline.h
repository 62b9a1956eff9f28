/* Multi-rank nested pipeline schedule and its replay (host only, no GPU work).
 *
 * Sec. 3.1 of the paper: the LLM runs a pipeline schedule over P ranks (classic 1F1B, or
 * the interleaved order with V model chunks per rank); encoder and generator work is
 * grouped in units of P microbatches, one microbatch per rank, and the BuildSchedule
 * figure nests those units into the unchanged LLM schedule.  Sec. 2.2 "Performance
 * analysis" states what the replay is checked against: bubble rate (P-1)/(M+P-1) for
 * 1F1B, peak modality activations (M/P) A_m for the compute-efficient order, W units for
 * the nested one.
 *
 * Readings of what the paper leaves open: column j of the LLM schedule is the j-th LLM op
 * of every rank; rank r owns microbatch u*P + r of unit u; for rank r the LLM output of a
 * unit is ready when the last rank has forwarded that microbatch through the last chunk;
 * the encoder gradient of a unit is ready for all ranks when rank 0 has backed the unit's
 * last microbatch through chunk 0.  Pipeline position of chunk c on rank r is c*P + r.
 *
 * All pointers are host pointers owned by the caller.  Errors are return codes with a
 * message in bm_last_error(); nothing is allocated that outlives a call.
 */
#ifndef BIGMAC_PIPELINE_H
#define BIGMAC_PIPELINE_H

#include "bigmac_block.h"

#ifdef __cplusplus
extern "C" {
#endif

/* additional order for the pipeline functions: encoder inside the first-position forward /
 * backward on rank 0, generator inside the last-position forward on rank P-1 (Sec. 2.2
 * "Memory-efficient systems") */
enum { BM_ORDER_MEMORY_EFFICIENT = 3 };

typedef struct {
  int32_t op;      /* BM_OP_*                                                     */
  int32_t index;   /* microbatch for LLM ops, unit for encoder / generator ops    */
  int32_t chunk;   /* model chunk of an LLM op, 0 otherwise                       */
  int32_t column;  /* LLM column the op belongs to (-1 for the encoder warm-up)   */
} bm_pipe_op;

/* LLM ops of one rank in execution order: 2*M*V ops.  V = 1: classic 1F1B (rank r warms
 * up P-r-1 forwards).  V >= 2: interleaved order (warm-up 2(P-r-1) + (V-1)P forwards; the
 * k-th forward slot runs chunk (k div P) mod V of microbatch (k div PV)*P + k mod P, the
 * backward slots walk the chunks in reverse).  M must be a multiple of P.
 * n_ops: in = capacity of ops, out = ops written (or needed, with BM_ERR_INVALID_ARG). */
bm_status bm_pipeline_llm_schedule(int32_t P, int32_t V, int32_t M, int32_t rank,
                                   bm_pipe_op* ops, int32_t* n_ops);

/* Program of one rank for `order` (BM_ORDER_NESTED, BM_ORDER_COMPUTE_EFFICIENT or
 * BM_ORDER_MEMORY_EFFICIENT): its LLM ops, unchanged, with the unit ops nested.  At most
 * 2*M*V + 4*M/P ops. */
bm_status bm_pipeline_build_schedule(int32_t order, int32_t P, int32_t V, int32_t M, int32_t W,
                                     int32_t has_generator, int32_t rank,
                                     bm_pipe_op* ops, int32_t* n_ops);

typedef struct {
  int32_t order, P, V, M, W, has_generator;
  const double* llm_fwd;   /* [P*V] seconds of one microbatch through (rank, chunk), rank*V + chunk */
  const double* llm_bwd;   /* [P*V]                                                                 */
  const double* enc_fwd;   /* [M] seconds of the encoder forward of each microbatch                  */
  const double* enc_bwd;   /* [M]                                                                    */
  const double* gen_fwd;   /* [M] (ignored without generator, may be NULL)                           */
  const double* gen_bwd;   /* [M]                                                                    */
  double p2p;              /* seconds added to every edge that crosses ranks                         */
  double act_llm;          /* bytes one (microbatch, chunk) keeps from its forward to its backward   */
  const double* act_enc;   /* [M] bytes kept from encoder forward to encoder backward, or NULL       */
  const double* act_gen;   /* [M] bytes kept from generator forward to generator backward, or NULL   */
} bm_pipe_replay_config;

typedef struct {
  double makespan;         /* seconds until the last rank finishes                                   */
  double bubble;           /* 1 - sum(busy) / (P * makespan)                                         */
  double* busy;            /* [P] out: seconds each rank spent in operators                          */
  double* peak;            /* [P] out: activation high-water mark in bytes                           */
  double* peak_enc;        /* [P] out: encoder part                                                  */
  double* peak_gen;        /* [P] out: generator part                                                */
  double* peak_llm;        /* [P] out: LLM part                                                      */
} bm_pipe_replay_result;

/* Replays the P rank programs: an op starts when its rank is free and its inputs from
 * other ranks have arrived.  Returns BM_ERR_INVALID_ARG with "rank programs deadlock" when
 * no rank can advance (e.g. W too small for the LLM schedule).  Output arrays may be NULL. */
bm_status bm_pipeline_replay(const bm_pipe_replay_config* cfg, bm_pipe_replay_result* res);

/* ---- communication operators and the deadlock check (Sec. 3.1 "Communication operator",
 *      Sec. 3.2; the executor-interface figure names insert_comm_ops and deadlock_check) ----
 *
 * Every cross-rank data dependency of a compute op becomes a receive placed right before it,
 * every tensor another rank consumes a send placed right after it.  A message is identified
 * by (what, microbatch, edge); edges whose two ends sit on one rank need no message. */
enum { BM_OP_SEND = 6, BM_OP_RECV = 7 };
enum {
  BM_MSG_ACT = 0,    /* forward activation into pipeline position `edge`       (edge-1 -> edge)  */
  BM_MSG_GRAD = 1,   /* gradient of the input of pipeline position `edge`      (edge -> edge-1)  */
  BM_MSG_FEAT = 2,   /* encoder features of a microbatch to the entry rank     (m mod P -> 0)    */
  BM_MSG_FGRAD = 3,  /* input-embedding gradient back to the encoder owner     (0 -> m mod P)    */
  BM_MSG_OUT = 4,    /* LLM output of a microbatch to its generator owner      (P-1 -> m mod P)  */
  BM_MSG_OGRAD = 5   /* generator-input gradient back to the exit rank         (m mod P -> P-1)  */
};

typedef struct {
  int32_t op;      /* BM_OP_* (compute) or BM_OP_SEND / BM_OP_RECV                          */
  int32_t index;   /* compute: microbatch or unit;  message: microbatch                     */
  int32_t chunk;   /* compute: model chunk;         message: edge (a pipeline position)     */
  int32_t peer;    /* message: the other rank; -1 for compute ops                           */
  int32_t what;    /* message: BM_MSG_*;       -1 for compute ops                           */
} bm_pipe_xop;

/* Program of one rank with its communication operators: at most 3 ops per compute op. */
bm_status bm_pipeline_comm_schedule(int32_t order, int32_t P, int32_t V, int32_t M, int32_t W,
                                    int32_t has_generator, int32_t rank,
                                    bm_pipe_xop* ops, int32_t* n_ops);

typedef struct {
  int32_t deadlock;      /* 1: some rank can never advance (also: a compute op placed before the
                            op of its own rank that produces its input)                       */
  int32_t unmatched;     /* sends without a receive + receives without a send + duplicates    */
  int32_t fifo;          /* 1: on every ordered pair of ranks messages are received in the order
                            they were sent (enough for a transport that matches by order)     */
  int32_t max_inflight;  /* most messages posted but not yet received on one ordered pair     */
  int64_t messages;      /* sends over all ranks                                              */
} bm_pipe_comm_report;

/* Runs the P programs with sends that never block and receives that block until their send
 * was posted (the executor waits on receive handles before consuming, Sec. 3.2). */
bm_status bm_pipeline_check_comm(int32_t order, int32_t P, int32_t V, int32_t M, int32_t W,
                                 int32_t has_generator, bm_pipe_comm_report* report);

#ifdef __cplusplus
}
#endif
#endif
