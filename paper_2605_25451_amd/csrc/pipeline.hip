// Multi-rank nested pipeline schedule and its replay (host code only).
//
// Sec. 3.1 of the paper nests encoder / generator units of P microbatches into an
// unchanged LLM pipeline schedule (BuildSchedule figure); Sec. 2.2 "Performance
// analysis" gives the bubble and memory figures of the two baseline orders.  This
// file generates the rank programs (classic and interleaved 1F1B, the nested, the
// compute-efficient and the memory-efficient order) and replays them with given
// operator durations: an op starts when its rank is free and its cross-rank inputs
// have arrived.
//
// Slot arithmetic: a rank's LLM program is fully described by its warm-up count w:
// forward slot k sits at program position k (k < w) or w + 2(k-w); backward slot k
// at w + 2k + 1 while forwards remain, then contiguously.  Slot k maps to
// (microbatch, chunk) by the interleaving rule in the header.
#include "common.h"

#include "../../include/bigmac_pipeline.h"

#include <vector>

namespace {

struct Shape {
  int P, V, M;
  int U() const { return M / P; }
  int slots() const { return M * V; }
  int warmup(int rank) const {
    int w = V == 1 ? P - rank - 1 : 2 * (P - rank - 1) + (V - 1) * P;
    return w < slots() ? w : slots();
  }
  int slot_mb(int k) const { return (k / (P * V)) * P + k % P; }
  int slot_chunk_fwd(int k) const { return (k / P) % V; }
  int slot_chunk_bwd(int k) const { return V - 1 - (k / P) % V; }
};

// LLM op at program position j of a rank with warm-up w
bm_pipe_op llm_op_at(const Shape& s, int w, int j) {
  const int n = s.slots();
  bm_pipe_op op;
  op.column = j;
  bool fwd;
  int k;
  if (j < w) { fwd = true; k = j; }
  else if (j < w + 2 * (n - w)) { fwd = ((j - w) & 1) == 0; k = fwd ? w + (j - w) / 2 : (j - w) / 2; }
  else { fwd = false; k = (n - w) + (j - w - 2 * (n - w)); }
  op.op = fwd ? BM_OP_LLM_FWD : BM_OP_LLM_BWD;
  op.index = s.slot_mb(k);
  op.chunk = fwd ? s.slot_chunk_fwd(k) : s.slot_chunk_bwd(k);
  return op;
}

bm_status check_shape(int P, int V, int M, int rank) {
  BM_ARG_CHECK(P >= 1 && V >= 1 && M >= 1, "pipeline: P=%d V=%d M=%d must be positive", P, V, M);
  BM_ARG_CHECK(M % P == 0, "pipeline: M=%d must be a multiple of P=%d", M, P);
  BM_ARG_CHECK(rank >= 0 && rank < P, "pipeline: rank %d outside [0,%d)", rank, P);
  BM_ARG_CHECK((long)M * V <= (1 << 24), "pipeline: M*V too large");
  return BM_OK;
}

void build_program(const Shape& s, int order, int W, bool gen, int rank, std::vector<bm_pipe_op>& out) {
  out.clear();
  const int n = 2 * s.slots();
  const int w_self = s.warmup(rank), w_first = s.warmup(0), w_last = s.warmup(s.P - 1);
  if (order == BM_ORDER_MEMORY_EFFICIENT) {
    for (int j = 0; j < n; ++j) out.push_back(llm_op_at(s, w_self, j));
    return;
  }
  const int U = s.U();
  int next_unit = 0;
  const int warm_units = order == BM_ORDER_COMPUTE_EFFICIENT ? U : (W < U ? W : U);
  for (; next_unit < warm_units; ++next_unit) out.push_back({BM_OP_ENC_FWD, next_unit, 0, -1});
  for (int j = 0; j < n; ++j) {
    out.push_back(llm_op_at(s, w_self, j));
    // only the entry rank's and the exit rank's ops of this column can trigger unit ops;
    // entry-rank triggers come first (rank order within a column)
    const bm_pipe_op first = llm_op_at(s, w_first, j);
    if (order == BM_ORDER_NESTED && first.op == BM_OP_LLM_BWD && first.chunk == 0 &&
        first.index % s.P == s.P - 1) {
      out.push_back({BM_OP_ENC_BWD, first.index / s.P, 0, j});
      if (next_unit < U) out.push_back({BM_OP_ENC_FWD, next_unit++, 0, j});
    }
    const bm_pipe_op last = llm_op_at(s, w_last, j);
    if (gen && last.op == BM_OP_LLM_FWD && last.chunk == s.V - 1 && last.index % s.P == rank) {
      out.push_back({BM_OP_GEN_FWD, last.index / s.P, 0, j});
      out.push_back({BM_OP_GEN_BWD, last.index / s.P, 0, j});
    }
  }
  if (order == BM_ORDER_COMPUTE_EFFICIENT)
    for (int u = 0; u < U; ++u) out.push_back({BM_OP_ENC_BWD, u, 0, n});
}

bm_status emit(const std::vector<bm_pipe_op>& prog, bm_pipe_op* ops, int32_t* n_ops) {
  BM_ARG_CHECK(n_ops != nullptr, "pipeline: n_ops is NULL");
  const int32_t cap = *n_ops;
  *n_ops = (int32_t)prog.size();
  BM_ARG_CHECK(ops != nullptr && cap >= (int32_t)prog.size(), "pipeline: %zu ops need more than the %d given",
               prog.size(), cap);
  for (size_t i = 0; i < prog.size(); ++i) ops[i] = prog[i];
  return BM_OK;
}

// finish times of everything a rank may wait for; a negative value = not finished yet
struct Finish {
  Shape s;
  std::vector<double> llm;    // [rank][fwd/bwd][mb][chunk]
  std::vector<double> unit;   // [rank][op kind 0..3: E e G H][unit]
  explicit Finish(const Shape& sh) : s(sh), llm((size_t)sh.P * 2 * sh.M * sh.V, -1.0),
                                     unit((size_t)sh.P * 4 * sh.U(), -1.0) {}
  double& at_llm(int rank, bool bwd, int mb, int chunk) {
    return llm[(((size_t)rank * 2 + (bwd ? 1 : 0)) * s.M + mb) * s.V + chunk];
  }
  double& at_unit(int rank, int kind, int u) { return unit[((size_t)rank * 4 + kind) * s.U() + u]; }
};

// ---- communication operators ----------------------------------------------------------------
bm_pipe_xop compute_xop(const bm_pipe_op& op) { return {op.op, op.index, op.chunk, -1, -1}; }
bm_pipe_xop message(int dir, int peer, int what, int mb, int edge) { return {dir, mb, edge, peer, what}; }

void build_comm_program(const Shape& s, int order, int W, bool gen, int rank, std::vector<bm_pipe_xop>& out) {
  std::vector<bm_pipe_op> prog;
  build_program(s, order, W, gen, rank, prog);
  out.clear();
  const int P = s.P, r = rank, last = s.P * s.V - 1;
  const bool fused = order == BM_ORDER_MEMORY_EFFICIENT;
  for (const bm_pipe_op& op : prog) {
    bm_pipe_xop pre[2], post[2];
    int npre = 0, npost = 0;
    const int i = op.index;
    if (op.op == BM_OP_LLM_FWD || op.op == BM_OP_LLM_BWD) {
      const int pos = op.chunk * P + r;
      const int up = (pos + P - 1) % P, down = (pos + 1) % P;   // ranks of the neighbouring positions
      if (op.op == BM_OP_LLM_FWD) {
        if (pos > 0 && up != r) pre[npre++] = message(BM_OP_RECV, up, BM_MSG_ACT, i, pos);
        if (pos == 0 && !fused && i % P != r) pre[npre++] = message(BM_OP_RECV, i % P, BM_MSG_FEAT, i, 0);
        if (pos < last && down != r) post[npost++] = message(BM_OP_SEND, down, BM_MSG_ACT, i, pos + 1);
        if (pos == last && gen && !fused && i % P != r) post[npost++] = message(BM_OP_SEND, i % P, BM_MSG_OUT, i, last);
      } else {
        if (pos < last && down != r) pre[npre++] = message(BM_OP_RECV, down, BM_MSG_GRAD, i, pos + 1);
        if (pos == last && gen && !fused && i % P != r) pre[npre++] = message(BM_OP_RECV, i % P, BM_MSG_OGRAD, i, last);
        if (pos > 0 && up != r) post[npost++] = message(BM_OP_SEND, up, BM_MSG_GRAD, i, pos);
        if (pos == 0 && !fused && i % P != r) post[npost++] = message(BM_OP_SEND, i % P, BM_MSG_FGRAD, i, 0);
      }
    } else {
      const int m = i * P + r;
      if (op.op == BM_OP_ENC_FWD && r != 0) post[npost++] = message(BM_OP_SEND, 0, BM_MSG_FEAT, m, 0);
      if (op.op == BM_OP_ENC_BWD && r != 0) pre[npre++] = message(BM_OP_RECV, 0, BM_MSG_FGRAD, m, 0);
      if (op.op == BM_OP_GEN_FWD && r != P - 1) pre[npre++] = message(BM_OP_RECV, P - 1, BM_MSG_OUT, m, last);
      if (op.op == BM_OP_GEN_BWD && r != P - 1) post[npost++] = message(BM_OP_SEND, P - 1, BM_MSG_OGRAD, m, last);
    }
    for (int k = 0; k < npre; ++k) out.push_back(pre[k]);
    out.push_back(compute_xop(op));
    for (int k = 0; k < npost; ++k) out.push_back(post[k]);
  }
}

// dense index of a message (what, microbatch, edge): the key under which sends and receives meet
struct MessageIndex {
  int M, edges;
  size_t size() const { return (size_t)6 * M * edges; }
  size_t at(int what, int mb, int edge) const { return ((size_t)what * M + mb) * edges + edge; }
};

int unit_kind(int opcode) {
  switch (opcode) {
    case BM_OP_ENC_FWD: return 0;
    case BM_OP_ENC_BWD: return 1;
    case BM_OP_GEN_FWD: return 2;
    default: return 3;
  }
}

}  // namespace

extern "C" bm_status bm_pipeline_llm_schedule(int32_t P, int32_t V, int32_t M, int32_t rank,
                                              bm_pipe_op* ops, int32_t* n_ops) {
  BM_RETURN_IF(check_shape(P, V, M, rank));
  const Shape s{P, V, M};
  std::vector<bm_pipe_op> prog;
  const int w = s.warmup(rank);
  for (int j = 0; j < 2 * s.slots(); ++j) prog.push_back(llm_op_at(s, w, j));
  return emit(prog, ops, n_ops);
}

extern "C" bm_status bm_pipeline_build_schedule(int32_t order, int32_t P, int32_t V, int32_t M,
                                                int32_t W, int32_t has_generator, int32_t rank,
                                                bm_pipe_op* ops, int32_t* n_ops) {
  BM_RETURN_IF(check_shape(P, V, M, rank));
  BM_ARG_CHECK(order == BM_ORDER_NESTED || order == BM_ORDER_COMPUTE_EFFICIENT ||
               order == BM_ORDER_MEMORY_EFFICIENT, "pipeline: order %d", order);
  BM_ARG_CHECK(order != BM_ORDER_NESTED || W >= 1, "pipeline: W=%d must be at least 1", W);
  std::vector<bm_pipe_op> prog;
  build_program(Shape{P, V, M}, order, W, has_generator != 0, rank, prog);
  return emit(prog, ops, n_ops);
}

extern "C" bm_status bm_pipeline_comm_schedule(int32_t order, int32_t P, int32_t V, int32_t M, int32_t W,
                                               int32_t has_generator, int32_t rank, bm_pipe_xop* ops,
                                               int32_t* n_ops) {
  BM_RETURN_IF(check_shape(P, V, M, rank));
  BM_ARG_CHECK(order == BM_ORDER_NESTED || order == BM_ORDER_COMPUTE_EFFICIENT ||
               order == BM_ORDER_MEMORY_EFFICIENT, "pipeline: order %d", order);
  BM_ARG_CHECK(order != BM_ORDER_NESTED || W >= 1, "pipeline: W=%d must be at least 1", W);
  BM_ARG_CHECK(n_ops != nullptr, "pipeline: n_ops is NULL");
  std::vector<bm_pipe_xop> prog;
  build_comm_program(Shape{P, V, M}, order, W, has_generator != 0, rank, prog);
  const int32_t cap = *n_ops;
  *n_ops = (int32_t)prog.size();
  BM_ARG_CHECK(ops != nullptr && cap >= (int32_t)prog.size(), "pipeline: %zu ops need more than the %d given",
               prog.size(), cap);
  for (size_t i = 0; i < prog.size(); ++i) ops[i] = prog[i];
  return BM_OK;
}

extern "C" bm_status bm_pipeline_check_comm(int32_t order, int32_t P, int32_t V, int32_t M, int32_t W,
                                            int32_t has_generator, bm_pipe_comm_report* report) {
  BM_RETURN_IF(check_shape(P, V, M, 0));
  BM_ARG_CHECK(order == BM_ORDER_NESTED || order == BM_ORDER_COMPUTE_EFFICIENT ||
               order == BM_ORDER_MEMORY_EFFICIENT, "pipeline: order %d", order);
  BM_ARG_CHECK(order != BM_ORDER_NESTED || W >= 1, "pipeline: W=%d must be at least 1", W);
  BM_ARG_CHECK(report != nullptr, "pipeline: report is NULL");
  const Shape s{P, V, M};
  const bool gen = has_generator != 0, fused = order == BM_ORDER_MEMORY_EFFICIENT;
  const int last = P * V - 1;
  std::vector<std::vector<bm_pipe_xop>> prog(P);
  for (int r = 0; r < P; ++r) build_comm_program(s, order, W, gen, r, prog[r]);

  // matching: every message key is sent once and received once, between the same two ranks
  const MessageIndex mi{M, P * V};
  std::vector<int> n_send(mi.size(), 0), n_recv(mi.size(), 0), src(mi.size(), -1), dst(mi.size(), -1);
  int unmatched = 0;
  int64_t messages = 0;
  for (int r = 0; r < P; ++r)
    for (const bm_pipe_xop& op : prog[r]) {
      if (op.op != BM_OP_SEND && op.op != BM_OP_RECV) continue;
      const size_t k = mi.at(op.what, op.index, op.chunk);
      if (op.op == BM_OP_SEND) {
        ++messages;
        if (n_send[k]++ > 0 || (dst[k] >= 0 && dst[k] != op.peer) || (src[k] >= 0 && src[k] != r)) ++unmatched;
        src[k] = r; dst[k] = op.peer;
      } else {
        if (n_recv[k]++ > 0 || (src[k] >= 0 && src[k] != op.peer) || (dst[k] >= 0 && dst[k] != r)) ++unmatched;
        src[k] = op.peer; dst[k] = r;
      }
    }
  for (size_t k = 0; k < mi.size(); ++k) unmatched += n_send[k] > n_recv[k] ? n_send[k] - n_recv[k] : n_recv[k] - n_send[k];

  // run: sends never block, a receive waits for its send, a compute op for its local producers
  Finish ran(s);                                    // >= 0 marks a compute op that has run
  std::vector<char> posted(mi.size(), 0);
  std::vector<size_t> pc(P, 0);
  std::vector<int> inflight((size_t)P * P, 0);
  std::vector<std::vector<size_t>> sent_seq((size_t)P * P), recv_seq((size_t)P * P);
  int max_inflight = 0;
  size_t left = 0;
  for (int r = 0; r < P; ++r) left += prog[r].size();
  bool deadlock = false;
  auto ran_llm = [&](int r, bool bwd, int mb, int c) { return ran.at_llm(r, bwd, mb, c) >= 0.0; };
  auto ran_unit = [&](int r, int kind, int u) { return ran.at_unit(r, kind, u) >= 0.0; };
  while (left > 0) {
    bool moved = false;
    for (int r = 0; r < P; ++r) {
      while (pc[r] < prog[r].size()) {
        const bm_pipe_xop& op = prog[r][pc[r]];
        const int i = op.index, c = op.chunk;
        if (op.op == BM_OP_SEND) {
          posted[mi.at(op.what, i, c)] = 1;
          const size_t pair = (size_t)r * P + op.peer;
          max_inflight = ++inflight[pair] > max_inflight ? inflight[pair] : max_inflight;
          sent_seq[pair].push_back(mi.at(op.what, i, c));
        } else if (op.op == BM_OP_RECV) {
          if (!posted[mi.at(op.what, i, c)]) break;
          const size_t pair = (size_t)op.peer * P + r;
          --inflight[pair];
          recv_seq[pair].push_back(mi.at(op.what, i, c));
        } else {
          bool ok = true;
          const int pos = c * P + r;
          switch (op.op) {
            case BM_OP_LLM_FWD:
              if (pos > 0 && (pos - 1) % P == r) ok = ok && ran_llm(r, false, i, c - 1);
              if (pos == 0 && !fused && i % P == r) ok = ok && ran_unit(r, 0, i / P);
              break;
            case BM_OP_LLM_BWD:
              ok = ok && ran_llm(r, false, i, c);
              if (pos < last && (pos + 1) % P == r) ok = ok && ran_llm(r, true, i, c + 1);
              if (pos == last && gen && !fused && i % P == r) ok = ok && ran_unit(r, 3, i / P);
              break;
            case BM_OP_ENC_BWD:
              ok = ok && ran_unit(r, 0, i);
              if (r == 0) ok = ok && ran_llm(0, true, i * P, 0);
              break;
            case BM_OP_GEN_FWD:
              if (r == P - 1) ok = ok && ran_llm(r, false, i * P + r, V - 1);
              break;
            case BM_OP_GEN_BWD: ok = ok && ran_unit(r, 2, i); break;
            default: break;
          }
          if (!ok) break;
          if (op.op == BM_OP_LLM_FWD || op.op == BM_OP_LLM_BWD) ran.at_llm(r, op.op == BM_OP_LLM_BWD, i, c) = 1.0;
          else ran.at_unit(r, unit_kind(op.op), i) = 1.0;
        }
        ++pc[r];
        --left;
        moved = true;
      }
    }
    if (!moved) { deadlock = true; break; }
  }
  bool fifo = !deadlock;
  for (size_t pair = 0; pair < sent_seq.size() && fifo; ++pair) fifo = sent_seq[pair] == recv_seq[pair];
  report->deadlock = deadlock ? 1 : 0;
  report->unmatched = unmatched;
  report->fifo = fifo ? 1 : 0;
  report->max_inflight = max_inflight;
  report->messages = messages;
  return BM_OK;
}

extern "C" bm_status bm_pipeline_replay(const bm_pipe_replay_config* cfg, bm_pipe_replay_result* res) {
  BM_ARG_CHECK(cfg && res, "pipeline: NULL config or result");
  BM_RETURN_IF(check_shape(cfg->P, cfg->V, cfg->M, 0));
  const int order = cfg->order;
  BM_ARG_CHECK(order == BM_ORDER_NESTED || order == BM_ORDER_COMPUTE_EFFICIENT ||
               order == BM_ORDER_MEMORY_EFFICIENT, "pipeline: order %d", order);
  BM_ARG_CHECK(order != BM_ORDER_NESTED || cfg->W >= 1, "pipeline: W=%d must be at least 1", cfg->W);
  BM_ARG_CHECK(cfg->llm_fwd && cfg->llm_bwd && cfg->enc_fwd && cfg->enc_bwd, "pipeline: NULL duration arrays");
  const bool gen = cfg->has_generator != 0;
  BM_ARG_CHECK(!gen || (cfg->gen_fwd && cfg->gen_bwd), "pipeline: generator durations are NULL");
  const Shape s{cfg->P, cfg->V, cfg->M};
  const int P = s.P, V = s.V;
  const bool fused = order == BM_ORDER_MEMORY_EFFICIENT;
  const double lat = cfg->p2p;

  std::vector<std::vector<bm_pipe_op>> prog(P);
  for (int r = 0; r < P; ++r) build_program(s, order, cfg->W, gen, r, prog[r]);
  Finish fin(s);
  std::vector<size_t> pc(P, 0);
  std::vector<double> clock(P, 0.0), busy(P, 0.0);
  size_t left = 0;
  for (int r = 0; r < P; ++r) left += prog[r].size();

  // arrival time of a finished op's output at rank `to`, or -1 while it is unfinished
  auto arrival = [&](double t, int from, int to) { return t < 0.0 ? -1.0 : t + (from != to ? lat : 0.0); };

  while (left > 0) {
    bool moved = false;
    for (int r = 0; r < P; ++r) {
      while (pc[r] < prog[r].size()) {
        const bm_pipe_op op = prog[r][pc[r]];
        double need = 0.0;          // latest input arrival; -1 = some input is missing
        bool has_dep = false;
        double dep = 0.0, cost = 0.0;
        const int i = op.index, c = op.chunk;
        switch (op.op) {
          case BM_OP_LLM_FWD:
            cost = cfg->llm_fwd[r * V + c];
            if (r > 0) { has_dep = true; dep = arrival(fin.at_llm(r - 1, false, i, c), r - 1, r); }
            else if (c > 0) { has_dep = true; dep = arrival(fin.at_llm(P - 1, false, i, c - 1), P - 1, r); }
            else if (fused) cost += cfg->enc_fwd[i];
            else { has_dep = true; dep = arrival(fin.at_unit(i % P, 0, i / P), i % P, r); }
            if (fused && gen && r == P - 1 && c == V - 1) cost += cfg->gen_fwd[i] + cfg->gen_bwd[i];
            break;
          case BM_OP_LLM_BWD:
            cost = cfg->llm_bwd[r * V + c];
            if (r < P - 1) { has_dep = true; dep = arrival(fin.at_llm(r + 1, true, i, c), r + 1, r); }
            else if (c < V - 1) { has_dep = true; dep = arrival(fin.at_llm(0, true, i, c + 1), 0, r); }
            else if (gen && !fused) { has_dep = true; dep = arrival(fin.at_unit(i % P, 3, i / P), i % P, r); }
            if (fused && r == 0 && c == 0) cost += cfg->enc_bwd[i];
            break;
          case BM_OP_ENC_FWD: cost = cfg->enc_fwd[i * P + r]; break;
          case BM_OP_ENC_BWD:
            cost = cfg->enc_bwd[i * P + r];
            has_dep = true; dep = arrival(fin.at_llm(0, true, i * P + r, 0), 0, r);
            break;
          case BM_OP_GEN_FWD:
            cost = cfg->gen_fwd[i * P + r];
            has_dep = true; dep = arrival(fin.at_llm(P - 1, false, i * P + r, V - 1), P - 1, r);
            break;
          default: cost = cfg->gen_bwd[i * P + r]; break;
        }
        if (has_dep) {
          if (dep < 0.0) break;     // this rank waits
          need = dep;
        }
        const double start = clock[r] > need ? clock[r] : need;
        clock[r] = start + cost;
        busy[r] += cost;
        if (op.op == BM_OP_LLM_FWD || op.op == BM_OP_LLM_BWD) fin.at_llm(r, op.op == BM_OP_LLM_BWD, i, c) = clock[r];
        else fin.at_unit(r, unit_kind(op.op), i) = clock[r];
        ++pc[r];
        --left;
        moved = true;
      }
    }
    if (!moved) {
      bm::set_error("rank programs deadlock (W=%d too small for this LLM schedule?)", cfg->W);
      return BM_ERR_INVALID_ARG;
    }
  }
  double makespan = 0.0, total = 0.0;
  for (int r = 0; r < P; ++r) { makespan = clock[r] > makespan ? clock[r] : makespan; total += busy[r]; }
  res->makespan = makespan;
  res->bubble = makespan > 0.0 ? 1.0 - total / (P * makespan) : 0.0;

  // activation high-water marks: a function of each rank's program alone
  for (int r = 0; r < P; ++r) {
    double live_l = 0, live_e = 0, live_g = 0, pk = 0, pe = 0, pg = 0, pl = 0;
    auto ae = [&](int m) { return cfg->act_enc ? cfg->act_enc[m] : 0.0; };
    auto ag = [&](int m) { return cfg->act_gen ? cfg->act_gen[m] : 0.0; };
    for (const bm_pipe_op& op : prog[r]) {
      const int i = op.index, c = op.chunk;
      if (op.op == BM_OP_LLM_FWD) {
        live_l += cfg->act_llm;
        if (fused && r == 0 && c == 0) live_e += ae(i);
        if (fused && gen && r == P - 1 && c == V - 1) {   // generator lives inside this op
          pg = ag(i) > pg ? ag(i) : pg;
          const double t = live_l + live_e + live_g + ag(i);
          pk = t > pk ? t : pk;
        }
      } else if (op.op == BM_OP_ENC_FWD) live_e += ae(i * P + r);
      else if (op.op == BM_OP_GEN_FWD) live_g += ag(i * P + r);
      const double t = live_l + live_e + live_g;
      pk = t > pk ? t : pk; pe = live_e > pe ? live_e : pe; pg = live_g > pg ? live_g : pg;
      pl = live_l > pl ? live_l : pl;
      if (op.op == BM_OP_LLM_BWD) {
        live_l -= cfg->act_llm;
        if (fused && r == 0 && c == 0) live_e -= ae(i);
      } else if (op.op == BM_OP_ENC_BWD) live_e -= ae(i * P + r);
      else if (op.op == BM_OP_GEN_BWD) live_g -= ag(i * P + r);
    }
    if (res->busy) res->busy[r] = busy[r];
    if (res->peak) res->peak[r] = pk;
    if (res->peak_enc) res->peak_enc[r] = pe;
    if (res->peak_gen) res->peak_gen[r] = pg;
    if (res->peak_llm) res->peak_llm[r] = pl;
  }
  return BM_OK;
}
