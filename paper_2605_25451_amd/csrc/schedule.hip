// Host-side nested schedule (integer logic only).
//
// The nested order of Sec. 3.1 ("Compute operator", "Memory efficiency", the BuildSchedule
// figure) is produced here from the dependency rule the text states rather than by walking
// the printed loop: the LLM op sequence is fixed, and every encoder / generator op is placed
// at the first point of that sequence where what it consumes exists and what it needs is free:
//   - an encoder forward needs a free encoder slot (at most W units hold encoder activations);
//   - a generator forward+backward needs the LLM output of every microbatch of its unit;
//   - an encoder backward needs the LLM input gradient of every microbatch of its unit, and
//     frees the unit's slot, which the next pending encoder forward takes at once.
// Completion counters per unit decide readiness after each single LLM op.
//
// Reading for one pipeline stage acting as both entry and exit of the LLM: a unit is unit_size
// consecutive microbatches; the LLM order is 1F1B at unit granularity with llm_depth units in
// flight.  The compute-efficient order of Sec. 2.2 is the same placement with as many encoder
// slots as units and every encoder backward held back to the end.
#include "common.h"

#include <vector>

namespace {

struct Op { int32_t code, index; };

struct Units {
  int M, unit_size, U;
  int first(int u) const { return u * unit_size; }
  int last(int u) const { int e = (u + 1) * unit_size; return (e < M ? e : M) - 1; }
  int size(int u) const { return last(u) - first(u) + 1; }
  int of(int mb) const { return mb / unit_size; }
};

// One stage's 1F1B order as a flat op list: forward the next unit while fewer than `depth`
// units are in flight, otherwise back the oldest unit in flight.
std::vector<Op> llm_order(const Units& un, int depth) {
  std::vector<Op> ops;
  int forwarded = 0, backed = 0;
  while (backed < un.U) {
    const bool fwd = forwarded < un.U && forwarded - backed < depth;
    const int u = fwd ? forwarded++ : backed++;
    for (int mb = un.first(u); mb <= un.last(u); ++mb)
      ops.push_back({fwd ? BM_OP_LLM_FWD : BM_OP_LLM_BWD, mb});
  }
  return ops;
}

// Places encoder and generator ops into the LLM order.  enc_slots: units that may hold encoder
// activations at once; hold_enc_bwd: encoder backwards wait for the end of the LLM order.
// Returns false when an LLM forward comes up before its unit's encoder output can exist.
bool place(const Units& un, const std::vector<Op>& llm, int enc_slots, bool hold_enc_bwd, bool gen,
           std::vector<Op>& out) {
  std::vector<int> fwd_done(un.U, 0), bwd_done(un.U, 0);
  int live_enc = 0, next_enc = 0;
  auto fill_encoder_slots = [&] {
    while (live_enc < enc_slots && next_enc < un.U) { out.push_back({BM_OP_ENC_FWD, next_enc++}); ++live_enc; }
  };
  fill_encoder_slots();
  for (const Op& op : llm) {
    const int u = un.of(op.index);
    if (op.code == BM_OP_LLM_FWD) {
      if (u >= next_enc) return false;               // its encoder unit has not run
      out.push_back(op);
      if (++fwd_done[u] == un.size(u) && gen) {      // the unit's LLM output is complete
        out.push_back({BM_OP_GEN_FWD, u});
        out.push_back({BM_OP_GEN_BWD, u});
      }
    } else {
      out.push_back(op);
      if (++bwd_done[u] == un.size(u) && !hold_enc_bwd) {   // the unit's input gradient is complete
        out.push_back({BM_OP_ENC_BWD, u});
        --live_enc;
        fill_encoder_slots();
      }
    }
  }
  if (hold_enc_bwd)
    for (int u = 0; u < un.U; ++u) out.push_back({BM_OP_ENC_BWD, u});
  return true;
}

bool build(int order, const Units& un, int W, int depth, bool gen, std::vector<Op>& out) {
  if (order == BM_ORDER_SEQUENTIAL)                  // one unit in flight everywhere
    return place(un, llm_order(un, 1), 1, false, gen, out);
  if (order == BM_ORDER_COMPUTE_EFFICIENT)
    return place(un, llm_order(un, depth), un.U, true, gen, out);
  return place(un, llm_order(un, depth), W, false, gen, out);
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
  std::vector<Op> ops;
  if (!build(order, un, W, llm_depth, has_generator != 0, ops)) {
    set_error("bm_build_schedule: an LLM forward would run before its encoder unit (W=%d, %d units in flight)",
              W, llm_depth);
    return BM_ERR_INVALID_ARG;
  }
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
