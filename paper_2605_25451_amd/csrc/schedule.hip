// Host-side nested schedule (integer logic only).
//
// The nested order follows the paper's BuildSchedule algorithm (Sec. 3.1,
// "Memory efficiency" and the BuildSchedule figure): the LLM schedule is kept
// as given; W encoder-forward units are warmed up; after each LLM column the
// generator runs forward+backward for a unit whose LLM output just completed,
// and the encoder runs backward -- followed at once by the next pending
// encoder forward -- for a unit whose input gradient just completed.
//
// Reading for one pipeline stage acting as both entry and exit of the LLM: a
// unit is unit_size consecutive microbatches; the LLM schedule is 1F1B at unit
// granularity with llm_depth units in flight; a unit's LLM output is complete
// at the forward of its last microbatch, its encoder gradient at the backward
// of its last microbatch.
#include "common.h"

#include <vector>

namespace {

struct Op { int32_t code, index; };

struct Units {
  int M, unit_size, U;
  int first(int u) const { return u * unit_size; }
  int last(int u) const { int e = (u + 1) * unit_size; return (e < M ? e : M) - 1; }
  int of(int mb) const { return mb / unit_size; }
};

// columns of the 1F1B order: (is_backward, unit)
std::vector<std::pair<bool, int>> llm_columns(const Units& un, int depth) {
  std::vector<std::pair<bool, int>> cols;
  int warm = depth < un.U ? depth : un.U;
  for (int u = 0; u < warm; ++u) cols.push_back({false, u});
  int next_f = warm;
  for (int u = 0; u < un.U; ++u) {
    cols.push_back({true, u});
    if (next_f < un.U) cols.push_back({false, next_f++});
  }
  return cols;
}

void emit_column(std::vector<Op>& out, const Units& un, bool bwd, int u) {
  for (int mb = un.first(u); mb <= un.last(u); ++mb)
    out.push_back({bwd ? BM_OP_LLM_BWD : BM_OP_LLM_FWD, mb});
}

std::vector<Op> build(int order, const Units& un, int W, int depth, bool gen) {
  std::vector<Op> out;
  if (order == BM_ORDER_SEQUENTIAL) {
    for (int u = 0; u < un.U; ++u) {
      out.push_back({BM_OP_ENC_FWD, u});
      emit_column(out, un, false, u);
      if (gen) { out.push_back({BM_OP_GEN_FWD, u}); out.push_back({BM_OP_GEN_BWD, u}); }
      emit_column(out, un, true, u);
      out.push_back({BM_OP_ENC_BWD, u});
    }
    return out;
  }
  const bool nested = order == BM_ORDER_NESTED;
  int next_enc = 0;
  const int warm = nested ? (W < un.U ? W : un.U) : un.U;
  while (next_enc < warm) out.push_back({BM_OP_ENC_FWD, next_enc++});
  for (auto& col : llm_columns(un, depth)) {
    const bool bwd = col.first;
    const int u = col.second;
    emit_column(out, un, bwd, u);
    // the column's last op completes the unit's LLM output (forward) or its
    // encoder-input gradient (backward)
    if (!bwd && gen) { out.push_back({BM_OP_GEN_FWD, u}); out.push_back({BM_OP_GEN_BWD, u}); }
    if (bwd && nested) {
      out.push_back({BM_OP_ENC_BWD, u});
      if (next_enc < un.U) out.push_back({BM_OP_ENC_FWD, next_enc++});
    }
  }
  if (!nested)
    for (int u = 0; u < un.U; ++u) out.push_back({BM_OP_ENC_BWD, u});
  return out;
}

}  // namespace

using namespace bm;

extern "C" bm_status bm_build_schedule(int32_t order, int32_t M, int32_t unit_size, int32_t W,
                                       int32_t llm_depth, int32_t has_generator, int32_t* ops_out,
                                       int32_t* n_ops) {
  BM_ARG_CHECK(order >= 0 && order <= 2, "bm_build_schedule: order %d", order);
  BM_ARG_CHECK(M >= 1 && unit_size >= 1 && W >= 1 && llm_depth >= 1,
               "bm_build_schedule: M, unit_size, W, llm_depth must be >= 1");
  BM_ARG_CHECK(n_ops != nullptr, "bm_build_schedule: n_ops is NULL");
  Units un{M, unit_size, (M + unit_size - 1) / unit_size};
  BM_ARG_CHECK(order != BM_ORDER_NESTED || W >= (llm_depth < un.U ? llm_depth : un.U),
               "bm_build_schedule: W=%d encoder units cannot feed an LLM order with %d units in flight",
               W, llm_depth);
  std::vector<Op> ops = build(order, un, W, llm_depth, has_generator != 0);
  const int32_t cap = *n_ops;
  *n_ops = (int32_t)ops.size();
  if (cap < (int32_t)ops.size() || !ops_out) {
    set_error("bm_build_schedule: %zu ops needed, capacity %d", ops.size(), cap);
    return BM_ERR_INVALID_ARG;
  }
  for (size_t i = 0; i < ops.size(); ++i) { ops_out[2 * i] = ops[i].code; ops_out[2 * i + 1] = ops[i].index; }
  return BM_OK;
}

extern "C" bm_status bm_check_schedule(const int32_t* ops, int32_t n_ops, int32_t M,
                                       int32_t unit_size, int32_t has_generator, int32_t* peak_out) {
  BM_ARG_CHECK(ops && n_ops >= 0 && M >= 1 && unit_size >= 1, "bm_check_schedule: bad arguments");
  Units un{M, unit_size, (M + unit_size - 1) / unit_size};
  std::vector<int> enc_f(un.U, -1), enc_b(un.U, -1), gen_f(un.U, -1), gen_b(un.U, -1);
  std::vector<int> llm_f(M, -1), llm_b(M, -1);
  int live_e = 0, live_g = 0, live_l = 0, pe = 0, pg = 0, pl = 0;
  for (int i = 0; i < n_ops; ++i) {
    const int code = ops[2 * i], idx = ops[2 * i + 1];
    const bool unit_op = code == BM_OP_ENC_FWD || code == BM_OP_ENC_BWD || code == BM_OP_GEN_FWD ||
                         code == BM_OP_GEN_BWD;
    BM_ARG_CHECK(code >= 0 && code <= 5, "op %d: unknown opcode %d", i, code);
    BM_ARG_CHECK(idx >= 0 && idx < (unit_op ? un.U : M), "op %d: index %d out of range", i, idx);
    BM_ARG_CHECK(has_generator || (code != BM_OP_GEN_FWD && code != BM_OP_GEN_BWD),
                 "op %d: generator op in a schedule without generator", i);
    std::vector<int>* slot = code == BM_OP_ENC_FWD ? &enc_f : code == BM_OP_ENC_BWD ? &enc_b
                           : code == BM_OP_GEN_FWD ? &gen_f : code == BM_OP_GEN_BWD ? &gen_b
                           : code == BM_OP_LLM_FWD ? &llm_f : &llm_b;
    BM_ARG_CHECK((*slot)[idx] < 0, "op %d: opcode %d index %d appears twice", i, code, idx);
    (*slot)[idx] = i;
    switch (code) {
      case BM_OP_ENC_FWD: ++live_e; break;
      case BM_OP_ENC_BWD:
        BM_ARG_CHECK(enc_f[idx] >= 0, "op %d: encoder backward of unit %d before its forward", i, idx);
        BM_ARG_CHECK(llm_b[un.last(idx)] >= 0 && llm_b[un.first(idx)] >= 0,
                     "op %d: encoder backward of unit %d before its LLM backward", i, idx);
        for (int mb = un.first(idx); mb <= un.last(idx); ++mb)
          BM_ARG_CHECK(llm_b[mb] >= 0, "op %d: encoder backward of unit %d before LLM backward of microbatch %d", i, idx, mb);
        --live_e; break;
      case BM_OP_LLM_FWD:
        BM_ARG_CHECK(enc_f[un.of(idx)] >= 0, "op %d: LLM forward of microbatch %d before its encoder unit", i, idx);
        ++live_l; break;
      case BM_OP_LLM_BWD:
        BM_ARG_CHECK(llm_f[idx] >= 0, "op %d: LLM backward of microbatch %d before its forward", i, idx);
        BM_ARG_CHECK(!has_generator || gen_b[un.of(idx)] >= 0,
                     "op %d: LLM backward of microbatch %d before its generator backward", i, idx);
        --live_l; break;
      case BM_OP_GEN_FWD:
        for (int mb = un.first(idx); mb <= un.last(idx); ++mb)
          BM_ARG_CHECK(llm_f[mb] >= 0, "op %d: generator forward of unit %d before LLM forward of microbatch %d", i, idx, mb);
        ++live_g; break;
      case BM_OP_GEN_BWD:
        BM_ARG_CHECK(gen_f[idx] >= 0, "op %d: generator backward of unit %d before its forward", i, idx);
        --live_g; break;
    }
    pe = live_e > pe ? live_e : pe; pg = live_g > pg ? live_g : pg; pl = live_l > pl ? live_l : pl;
  }
  for (int u = 0; u < un.U; ++u) {
    BM_ARG_CHECK(enc_f[u] >= 0 && enc_b[u] >= 0, "unit %d: encoder op missing", u);
    BM_ARG_CHECK(!has_generator || (gen_f[u] >= 0 && gen_b[u] >= 0), "unit %d: generator op missing", u);
  }
  for (int mb = 0; mb < M; ++mb)
    BM_ARG_CHECK(llm_f[mb] >= 0 && llm_b[mb] >= 0, "microbatch %d: LLM op missing", mb);
  if (peak_out) { peak_out[0] = pe; peak_out[1] = pg; peak_out[2] = pl; }
  return BM_OK;
}
