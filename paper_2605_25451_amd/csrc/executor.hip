// Single-GPU micro-unit executor: interprets the op stream of the nested schedule
// (Sec. 3.2 "Pipeline Executor": opcode interpreter, runtime buffers keyed by
// microbatch / unit, module handoff with free-on-backward), with every compute op
// expanded into block forward/backward calls and the handoff kernels.  Host code only;
// all device work is enqueued on one stream in op order, so the op stream's
// dependency order is the execution order.
#include "common.h"

#include <vector>

using namespace bm;

namespace {

struct EncSlot { std::vector<char*> act, saved; char *feat, *dfeat; };
struct LlmSlot { std::vector<char*> act, saved; char* x_in; char* dh_out; };
struct GenSet  { std::vector<char*> act, saved, dcond; char *cond, *hsel, *dhsel, *dout; };

size_t saved_bytes(const bm_block_desc& d, int T, int S, int maxlen) {
  size_t sv = 0, sc = 0;
  bm_block_sizes(&d, T, S, maxlen < 1 ? 1 : maxlen, &sv, &sc);
  return sv;
}
size_t scratch_bytes_of(const bm_block_desc& d, int T, int S) {
  size_t sv = 0, sc = 0;
  bm_block_sizes(&d, T, S, T, &sv, &sc);
  return sc;
}
int max_len(const int32_t* cu, int S) {
  int m = 1;
  for (int s = 0; s < S; ++s) { int L = cu[s + 1] - cu[s]; m = L > m ? L : m; }
  return m;
}

struct Sizes {
  int maxT_llm = 1, maxS_llm = 1, maxT_enc = 1, maxS_enc = 1, maxT_gen = 1;
  size_t enc_slot = 0, llm_slot = 0, gen_set = 0, scratch = 0, ping = 0, total = 0;
};

}  // namespace

struct bm_executor {
  bm_executor_config cfg;
  std::vector<bm_block_params> enc_w, llm_w, gen_w, enc_g, llm_g, gen_g;
  void *proj_in = nullptr, *proj_out = nullptr;
  float *g_proj_in = nullptr, *g_proj_out = nullptr;
  std::vector<bm_microbatch> mbs;
  std::vector<bm_unit> units;
  int U = 0;
  size_t es = 2;
  Sizes sz;
  char* scratch = nullptr;
  char *ping[2] = {nullptr, nullptr};
  std::vector<EncSlot> enc_slots;
  std::vector<LlmSlot> llm_slots;
  GenSet gen;
  std::vector<int> enc_slot_of, llm_slot_of;      // unit / microbatch -> slot or -1
  std::vector<char> enc_busy, llm_busy;
  std::vector<int32_t> ops;
  size_t live = 0, peak = 0, live_enc = 0, peak_enc = 0;
  bool has_gen() const { return cfg.n_gen_blocks > 0; }
  int unit_first(int u) const { return u * cfg.unit_size; }
  int unit_last(int u) const { int e = (u + 1) * cfg.unit_size; return (e < cfg.M ? e : cfg.M) - 1; }
};

namespace {

// bytes of one live encoder unit / LLM microbatch / generator unit (actual sizes)
size_t enc_unit_bytes(const bm_executor& ex, int u) {
  const bm_unit& un = ex.units[u];
  const int ml = max_len(un.cu_host, un.S);
  size_t b = 0;
  for (int i = 0; i < ex.cfg.n_enc_blocks; ++i)
    b += saved_bytes(ex.cfg.enc, un.T, un.S, ml) + (size_t)un.T * ex.cfg.enc.hidden * ex.es;
  b += 2 * (size_t)un.T * ex.cfg.llm.hidden * ex.es;                 // feat, dfeat
  return b;
}
size_t llm_mb_bytes(const bm_executor& ex, int m) {
  const bm_microbatch& mb = ex.mbs[m];
  const int ml = max_len(mb.cu_host, mb.S);
  size_t b = (size_t)mb.T * ex.cfg.llm.hidden * ex.es;                // embedded input
  for (int i = 0; i < ex.cfg.n_llm_blocks; ++i)
    b += saved_bytes(ex.cfg.llm, mb.T, mb.S, ml) + (size_t)mb.T * ex.cfg.llm.hidden * ex.es;
  if (ex.has_gen()) b += (size_t)mb.T * ex.cfg.llm.hidden * ex.es;    // generator's output gradient
  return b;
}
size_t gen_unit_bytes(const bm_executor& ex, int u) {
  const bm_unit& un = ex.units[u];
  const int Tg = un.S * ex.cfg.gen_tokens_per_image;
  size_t b = 0;
  for (int i = 0; i < ex.cfg.n_gen_blocks; ++i)
    b += saved_bytes(ex.cfg.gen, Tg, un.S, ex.cfg.gen_tokens_per_image) + (size_t)Tg * ex.cfg.gen.hidden * ex.es;
  b += (size_t)un.S * (ex.cfg.gen.hidden + ex.cfg.llm.hidden) * ex.es;
  return b;
}

bm_status check_config(const bm_executor_config* c, const bm_microbatch* mbs, const bm_unit* units) {
  BM_ARG_CHECK(c && mbs && units, "executor: NULL config, microbatches or units");
  BM_ARG_CHECK(c->M >= 1 && c->unit_size >= 1, "executor: M and unit_size must be >= 1");
  BM_ARG_CHECK(c->n_enc_blocks >= 1 && c->n_llm_blocks >= 1 && c->n_gen_blocks >= 0,
               "executor: block counts");
  BM_ARG_CHECK(c->enc.dtype == c->llm.dtype && (c->n_gen_blocks == 0 || c->gen.dtype == c->llm.dtype),
               "executor: all modules must use one dtype");
  BM_ARG_CHECK(c->n_gen_blocks == 0 || (c->gen.norm == BM_NORM_ADALN && c->gen_tokens_per_image >= 1),
               "executor: generator blocks must be adaLN blocks with gen_tokens_per_image >= 1");
  const int U = (c->M + c->unit_size - 1) / c->unit_size;
  for (int u = 0; u < U; ++u) {
    const bm_unit& un = units[u];
    BM_ARG_CHECK(un.T >= 1 && un.S >= 1 && un.cu_dev && un.cu_host && un.patches,
                 "executor: unit %d has no encoder tokens or NULL pointers", u);
    BM_ARG_CHECK(un.cu_host[0] == 0 && un.cu_host[un.S] == un.T, "executor: unit %d cu_seqlens", u);
    int rows = 0, imgs = 0;
    const int last = (u + 1) * c->unit_size < c->M ? (u + 1) * c->unit_size : c->M;
    for (int m = u * c->unit_size; m < last; ++m) { rows += mbs[m].n_image_rows; imgs += mbs[m].n_images; }
    BM_ARG_CHECK(rows == un.T, "executor: unit %d has %d encoder tokens but its microbatches place %d rows", u, un.T, rows);
    if (c->n_gen_blocks > 0) {
      BM_ARG_CHECK(imgs == un.S, "executor: unit %d has %d images but its microbatches list %d", u, un.S, imgs);
      BM_ARG_CHECK(un.gen_cu_dev && un.gen_cu_host && un.latents && un.targets, "executor: unit %d generator inputs are NULL", u);
      BM_ARG_CHECK(un.gen_cu_host[un.S] == un.S * c->gen_tokens_per_image, "executor: unit %d gen_cu_seqlens", u);
    }
  }
  for (int m = 0; m < c->M; ++m) {
    const bm_microbatch& mb = mbs[m];
    BM_ARG_CHECK(mb.T >= 1 && mb.S >= 1 && mb.cu_dev && mb.cu_host && mb.base, "executor: microbatch %d", m);
    BM_ARG_CHECK(mb.n_image_rows == 0 || mb.image_rows, "executor: microbatch %d image_rows is NULL", m);
    BM_ARG_CHECK(c->n_gen_blocks == 0 || mb.n_images == 0 || mb.image_last_row, "executor: microbatch %d image_last_row is NULL", m);
    BM_ARG_CHECK(c->n_gen_blocks > 0 || mb.out_grad, "executor: microbatch %d needs out_grad without a generator", m);
  }
  return BM_OK;
}

Sizes plan_sizes(const bm_executor_config& c, const bm_microbatch* mbs, const bm_unit* units,
                 int enc_slots, int llm_slots) {
  Sizes z;
  const size_t es = elt_size(c.llm.dtype);
  const int U = (c.M + c.unit_size - 1) / c.unit_size;
  int maxS_img = 1;
  for (int m = 0; m < c.M; ++m) { z.maxT_llm = mbs[m].T > z.maxT_llm ? mbs[m].T : z.maxT_llm; z.maxS_llm = mbs[m].S > z.maxS_llm ? mbs[m].S : z.maxS_llm; }
  for (int u = 0; u < U; ++u) { z.maxT_enc = units[u].T > z.maxT_enc ? units[u].T : z.maxT_enc; z.maxS_enc = units[u].S > z.maxS_enc ? units[u].S : z.maxS_enc; }
  maxS_img = z.maxS_enc;
  z.maxT_gen = maxS_img * (c.gen_tokens_per_image > 0 ? c.gen_tokens_per_image : 1);
  auto al = [](size_t v) { return align_up(v, 256); };
  // encoder slot
  z.enc_slot = 0;
  for (int i = 0; i < c.n_enc_blocks; ++i)
    z.enc_slot += al(saved_bytes(c.enc, z.maxT_enc, z.maxS_enc, z.maxT_enc)) + al((size_t)z.maxT_enc * c.enc.hidden * es);
  z.enc_slot += 2 * al((size_t)z.maxT_enc * c.llm.hidden * es);
  // LLM slot
  z.llm_slot = al((size_t)z.maxT_llm * c.llm.hidden * es);
  for (int i = 0; i < c.n_llm_blocks; ++i)
    z.llm_slot += al(saved_bytes(c.llm, z.maxT_llm, z.maxS_llm, z.maxT_llm)) + al((size_t)z.maxT_llm * c.llm.hidden * es);
  if (c.n_gen_blocks > 0) z.llm_slot += al((size_t)z.maxT_llm * c.llm.hidden * es);
  // generator working set
  z.gen_set = 0;
  if (c.n_gen_blocks > 0) {
    for (int i = 0; i < c.n_gen_blocks; ++i)
      z.gen_set += al(saved_bytes(c.gen, z.maxT_gen, maxS_img, c.gen_tokens_per_image)) +
                   al((size_t)z.maxT_gen * c.gen.hidden * es) + al((size_t)maxS_img * c.gen.hidden * es);
    z.gen_set += al((size_t)maxS_img * c.gen.hidden * es) + 2 * al((size_t)maxS_img * c.llm.hidden * es) +
                 al((size_t)z.maxT_gen * c.gen.hidden * es);
  }
  // scratch: block workspaces, projector split-K partials, loss partials; two ping-pong gradients.
  // A block's workspace is not monotone in the token count (a shorter contraction can be cut into
  // more k ranges, each with its own fp32 partial tile), so the largest pack alone does not bound
  // it: the maximum is taken over the shape of every unit and microbatch that will run.
  size_t sc = loss_scratch_bytes(), v;
  auto upto = [&](size_t b) { sc = b > sc ? b : sc; };
  for (int m = 0; m < c.M; ++m) upto(scratch_bytes_of(c.llm, mbs[m].T, mbs[m].S));
  for (int u = 0; u < U; ++u) {
    upto(scratch_bytes_of(c.enc, units[u].T, units[u].S));
    upto(gemm_scratch_bytes(GEMM_TN, c.llm.hidden, c.enc.hidden, units[u].T, c.llm.dtype));
    if (c.n_gen_blocks > 0) {
      const int tpi = c.gen_tokens_per_image > 0 ? c.gen_tokens_per_image : 1;
      upto(scratch_bytes_of(c.gen, units[u].S * tpi, units[u].S));
      upto(gemm_scratch_bytes(GEMM_TN, c.gen.hidden, c.llm.hidden, units[u].S, c.llm.dtype));
    }
  }
  z.scratch = al(sc);
  size_t pg = (size_t)z.maxT_llm * c.llm.hidden;
  v = (size_t)z.maxT_enc * c.enc.hidden; pg = v > pg ? v : pg;
  if (c.n_gen_blocks > 0) { v = (size_t)z.maxT_gen * c.gen.hidden; pg = v > pg ? v : pg; }
  z.ping = al(pg * es);
  z.total = z.scratch + 2 * z.ping + z.gen_set + (size_t)enc_slots * z.enc_slot + (size_t)llm_slots * z.llm_slot;
  return z;
}

void track(bm_executor* ex, long delta, bool enc) {
  ex->live = (size_t)((long)ex->live + delta);
  if (ex->live > ex->peak) ex->peak = ex->live;
  if (enc) {
    ex->live_enc = (size_t)((long)ex->live_enc + delta);
    if (ex->live_enc > ex->peak_enc) ex->peak_enc = ex->live_enc;
  }
}

// ---- ops -------------------------------------------------------------------
bm_status enc_fwd(bm_executor* ex, int u, hipStream_t st) {
  int slot = -1;
  for (size_t i = 0; i < ex->enc_busy.size(); ++i) if (!ex->enc_busy[i]) { slot = (int)i; break; }
  if (slot < 0) { set_error("executor: no free encoder slot for unit %d", u); return BM_ERR_WORKSPACE_TOO_SMALL; }
  ex->enc_busy[slot] = 1; ex->enc_slot_of[u] = slot;
  track(ex, (long)enc_unit_bytes(*ex, u), true);
  const bm_unit& un = ex->units[u];
  EncSlot& s = ex->enc_slots[slot];
  const int ml = max_len(un.cu_host, un.S);
  const void* in = un.patches;
  for (int b = 0; b < ex->cfg.n_enc_blocks; ++b) {
    BM_RETURN_IF(bm_block_forward(&ex->cfg.enc, &ex->enc_w[b], in, un.cu_dev, un.cu_host, un.S, un.T, ml,
                                  nullptr, s.act[b], s.saved[b], ex->scratch, ex->sz.scratch, st));
    in = s.act[b];
  }
  // encoder -> LLM projector
  GemmEpilogue none;
  return gemm(GEMM_NT, ex->cfg.enc.dtype, un.T, ex->cfg.llm.hidden, ex->cfg.enc.hidden, in, ex->cfg.enc.hidden,
              ex->proj_in, ex->cfg.enc.hidden, s.feat, ex->cfg.llm.hidden, none, nullptr, 0, st);
}

int rows_before(const bm_executor* ex, int m) {      // offset of microbatch m inside its unit's rows
  int off = 0;
  for (int k = ex->unit_first(m / ex->cfg.unit_size); k < m; ++k) off += ex->mbs[k].n_image_rows;
  return off;
}
int images_before(const bm_executor* ex, int m) {
  int off = 0;
  for (int k = ex->unit_first(m / ex->cfg.unit_size); k < m; ++k) off += ex->mbs[k].n_images;
  return off;
}

bm_status llm_fwd(bm_executor* ex, int m, hipStream_t st) {
  const int u = m / ex->cfg.unit_size;
  if (ex->enc_slot_of[u] < 0) { set_error("executor: LLM forward of microbatch %d before its encoder unit", m); return BM_ERR_INVALID_ARG; }
  int slot = -1;
  for (size_t i = 0; i < ex->llm_busy.size(); ++i) if (!ex->llm_busy[i]) { slot = (int)i; break; }
  if (slot < 0) { set_error("executor: no free LLM slot for microbatch %d", m); return BM_ERR_WORKSPACE_TOO_SMALL; }
  ex->llm_busy[slot] = 1; ex->llm_slot_of[m] = slot;
  track(ex, (long)llm_mb_bytes(*ex, m), false);
  const bm_microbatch& mb = ex->mbs[m];
  LlmSlot& s = ex->llm_slots[slot];
  const int d = ex->cfg.llm.hidden, dt = ex->cfg.llm.dtype;
  // embed_preprocess: text rows from `base`, image rows from the unit's projected features
  BM_CHECK_HIP(hipMemcpyAsync(s.x_in, mb.base, (size_t)mb.T * d * ex->es, hipMemcpyDeviceToDevice, st));
  const char* feat = ex->enc_slots[ex->enc_slot_of[u]].feat + (size_t)rows_before(ex, m) * d * ex->es;
  BM_RETURN_IF(row_scatter(dt, feat, mb.image_rows, s.x_in, mb.n_image_rows, d, st));
  const int ml = max_len(mb.cu_host, mb.S);
  const void* in = s.x_in;
  for (int b = 0; b < ex->cfg.n_llm_blocks; ++b) {
    BM_RETURN_IF(bm_block_forward(&ex->cfg.llm, &ex->llm_w[b], in, mb.cu_dev, mb.cu_host, mb.S, mb.T, ml,
                                  nullptr, s.act[b], s.saved[b], ex->scratch, ex->sz.scratch, st));
    in = s.act[b];
  }
  return BM_OK;
}

bm_status gen_fwd(bm_executor* ex, int u, float* loss, hipStream_t st) {
  const bm_unit& un = ex->units[u];
  const int dt = ex->cfg.gen.dtype, dl = ex->cfg.llm.hidden, dg = ex->cfg.gen.hidden;
  const int tpi = ex->cfg.gen_tokens_per_image, Tg = un.S * tpi;
  GenSet& g = ex->gen;
  track(ex, (long)gen_unit_bytes(*ex, u), false);
  // conditioning rows: LLM output at the row that closes each image span
  int img = 0;
  for (int m = ex->unit_first(u); m <= ex->unit_last(u); ++m) {
    if (ex->llm_slot_of[m] < 0) { set_error("executor: generator of unit %d before LLM forward of microbatch %d", u, m); return BM_ERR_INVALID_ARG; }
    const LlmSlot& ls = ex->llm_slots[ex->llm_slot_of[m]];
    BM_RETURN_IF(row_gather(dt, ls.act[ex->cfg.n_llm_blocks - 1], ex->mbs[m].image_last_row,
                            g.hsel + (size_t)img * dl * ex->es, ex->mbs[m].n_images, dl, st));
    img += ex->mbs[m].n_images;
  }
  GemmEpilogue none;
  BM_RETURN_IF(gemm(GEMM_NT, dt, un.S, dg, dl, g.hsel, dl, ex->proj_out, dl, g.cond, dg, none, nullptr, 0, st));
  const void* in = un.latents;
  for (int b = 0; b < ex->cfg.n_gen_blocks; ++b) {
    BM_RETURN_IF(bm_block_forward(&ex->cfg.gen, &ex->gen_w[b], in, un.gen_cu_dev, un.gen_cu_host, un.S, Tg, tpi,
                                  g.cond, g.act[b], g.saved[b], ex->scratch, ex->sz.scratch, st));
    in = g.act[b];
  }
  return mse_loss(dt, in, un.targets, g.dout, (long)Tg * dg, loss + u, ex->scratch, st);
}

bm_status gen_bwd(bm_executor* ex, int u, hipStream_t st) {
  const bm_unit& un = ex->units[u];
  const int dt = ex->cfg.gen.dtype, dl = ex->cfg.llm.hidden, dg = ex->cfg.gen.hidden;
  const int tpi = ex->cfg.gen_tokens_per_image, Tg = un.S * tpi;
  GenSet& g = ex->gen;
  const void* dy = g.dout;
  for (int b = ex->cfg.n_gen_blocks - 1; b >= 0; --b) {
    const void* x = b == 0 ? un.latents : g.act[b - 1];
    char* dx = ex->ping[b & 1];
    BM_RETURN_IF(bm_block_backward(&ex->cfg.gen, &ex->gen_w[b], x, dy, un.gen_cu_dev, un.gen_cu_host, un.S, Tg,
                                   tpi, g.cond, g.saved[b], dx, &ex->gen_g[b], g.dcond[b], ex->scratch,
                                   ex->sz.scratch, st));
    dy = dx;
    if (b != ex->cfg.n_gen_blocks - 1)
      BM_RETURN_IF(add_inplace(dt, g.dcond[ex->cfg.n_gen_blocks - 1], g.dcond[b], (long)un.S * dg, st));
  }
  char* dcond = g.dcond[ex->cfg.n_gen_blocks - 1];
  GemmEpilogue none;
  // cond = hsel proj_out^T
  BM_RETURN_IF(gemm(GEMM_TN, dt, dg, dl, un.S, dcond, dg, g.hsel, dl, ex->g_proj_out, dl, none, ex->scratch, ex->sz.scratch, st));
  BM_RETURN_IF(gemm(GEMM_NN, dt, un.S, dl, dg, dcond, dg, ex->proj_out, dl, g.dhsel, dl, none, nullptr, 0, st));
  int img = 0;
  for (int m = ex->unit_first(u); m <= ex->unit_last(u); ++m) {
    LlmSlot& ls = ex->llm_slots[ex->llm_slot_of[m]];
    const bm_microbatch& mb = ex->mbs[m];
    BM_RETURN_IF(fill_zero(ls.dh_out, align_up((size_t)mb.T * dl * ex->es, 16), st));
    BM_RETURN_IF(row_scatter(dt, g.dhsel + (size_t)img * dl * ex->es, mb.image_last_row, ls.dh_out, mb.n_images, dl, st));
    img += mb.n_images;
  }
  track(ex, -(long)gen_unit_bytes(*ex, u), false);
  return BM_OK;
}

bm_status llm_bwd(bm_executor* ex, int m, float* loss, hipStream_t st) {
  const int u = m / ex->cfg.unit_size;
  if (ex->llm_slot_of[m] < 0) { set_error("executor: LLM backward of microbatch %d before its forward", m); return BM_ERR_INVALID_ARG; }
  const bm_microbatch& mb = ex->mbs[m];
  LlmSlot& s = ex->llm_slots[ex->llm_slot_of[m]];
  const int d = ex->cfg.llm.hidden, dt = ex->cfg.llm.dtype, n = ex->cfg.n_llm_blocks;
  const int ml = max_len(mb.cu_host, mb.S);
  const void* dy = s.dh_out;
  if (!ex->has_gen()) {
    dy = mb.out_grad;
    BM_RETURN_IF(dot_loss(dt, s.act[n - 1], mb.out_grad, (long)mb.T * d, loss + m, ex->scratch, st));
  }
  for (int b = n - 1; b >= 0; --b) {
    const void* x = b == 0 ? s.x_in : s.act[b - 1];
    char* dx = ex->ping[b & 1];
    BM_RETURN_IF(bm_block_backward(&ex->cfg.llm, &ex->llm_w[b], x, dy, mb.cu_dev, mb.cu_host, mb.S, mb.T, ml,
                                   nullptr, s.saved[b], dx, &ex->llm_g[b], nullptr, ex->scratch, ex->sz.scratch, st));
    dy = dx;
  }
  // input-embedding gradient rows go back to the owning encoder unit
  char* dfeat = ex->enc_slots[ex->enc_slot_of[u]].dfeat + (size_t)rows_before(ex, m) * d * ex->es;
  BM_RETURN_IF(row_gather(dt, dy, mb.image_rows, dfeat, mb.n_image_rows, d, st));
  ex->llm_busy[ex->llm_slot_of[m]] = 0; ex->llm_slot_of[m] = -1;
  track(ex, -(long)llm_mb_bytes(*ex, m), false);
  return BM_OK;
}

bm_status enc_bwd(bm_executor* ex, int u, hipStream_t st) {
  if (ex->enc_slot_of[u] < 0) { set_error("executor: encoder backward of unit %d before its forward", u); return BM_ERR_INVALID_ARG; }
  const bm_unit& un = ex->units[u];
  EncSlot& s = ex->enc_slots[ex->enc_slot_of[u]];
  const int de = ex->cfg.enc.hidden, dl = ex->cfg.llm.hidden, dt = ex->cfg.enc.dtype, n = ex->cfg.n_enc_blocks;
  const int ml = max_len(un.cu_host, un.S);
  GemmEpilogue none;
  // feat = enc_out proj_in^T
  BM_RETURN_IF(gemm(GEMM_TN, dt, dl, de, un.T, s.dfeat, dl, s.act[n - 1], de, ex->g_proj_in, de, none, ex->scratch, ex->sz.scratch, st));
  char* dy = ex->ping[n & 1];
  BM_RETURN_IF(gemm(GEMM_NN, dt, un.T, de, dl, s.dfeat, dl, ex->proj_in, de, dy, de, none, nullptr, 0, st));
  for (int b = n - 1; b >= 0; --b) {
    const void* x = b == 0 ? un.patches : s.act[b - 1];
    char* dx = ex->ping[b & 1];
    BM_RETURN_IF(bm_block_backward(&ex->cfg.enc, &ex->enc_w[b], x, dy, un.cu_dev, un.cu_host, un.S, un.T, ml,
                                   nullptr, s.saved[b], dx, &ex->enc_g[b], nullptr, ex->scratch, ex->sz.scratch, st));
    dy = dx;
  }
  ex->enc_busy[ex->enc_slot_of[u]] = 0; ex->enc_slot_of[u] = -1;
  track(ex, -(long)enc_unit_bytes(*ex, u), true);
  return BM_OK;
}

}  // namespace

extern "C" bm_status bm_executor_arena_bytes(const bm_executor_config* cfg, const bm_microbatch* mbs,
                                             const bm_unit* units, int32_t enc_slots, int32_t llm_slots,
                                             size_t* bytes) {
  BM_RETURN_IF(check_config(cfg, mbs, units));
  BM_ARG_CHECK(enc_slots >= 1 && llm_slots >= 1 && bytes, "executor: slot counts must be >= 1");
  *bytes = plan_sizes(*cfg, mbs, units, enc_slots, llm_slots).total;
  return BM_OK;
}

extern "C" bm_status bm_executor_create(const bm_executor_config* cfg, const bm_executor_params* w,
                                        const bm_executor_params* grads, const bm_microbatch* mbs,
                                        const bm_unit* units, void* arena, size_t arena_bytes,
                                        int32_t enc_slots, int32_t llm_slots, bm_executor** out) {
  BM_RETURN_IF(check_config(cfg, mbs, units));
  BM_ARG_CHECK(w && grads && out && arena, "executor: NULL params, grads, arena or out");
  BM_ARG_CHECK(enc_slots >= 1 && llm_slots >= 1, "executor: slot counts must be >= 1");
  BM_ARG_CHECK(w->enc && w->llm && grads->enc && grads->llm && w->proj_in && grads->proj_in,
               "executor: encoder/LLM parameters or projector are NULL");
  BM_ARG_CHECK(cfg->n_gen_blocks == 0 || (w->gen && grads->gen && w->proj_out && grads->proj_out),
               "executor: generator parameters or projector are NULL");
  BM_ARG_CHECK((reinterpret_cast<uintptr_t>(arena) & 255) == 0, "executor: arena must be 256-byte aligned");
  Sizes z = plan_sizes(*cfg, mbs, units, enc_slots, llm_slots);
  if (z.total > arena_bytes) {
    set_error("executor: arena needs %zu bytes, got %zu", z.total, arena_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  bm_executor* ex = new bm_executor();
  ex->cfg = *cfg;
  ex->U = (cfg->M + cfg->unit_size - 1) / cfg->unit_size;
  ex->es = elt_size(cfg->llm.dtype);
  ex->sz = z;
  ex->enc_w.assign(w->enc, w->enc + cfg->n_enc_blocks); ex->enc_g.assign(grads->enc, grads->enc + cfg->n_enc_blocks);
  ex->llm_w.assign(w->llm, w->llm + cfg->n_llm_blocks); ex->llm_g.assign(grads->llm, grads->llm + cfg->n_llm_blocks);
  if (cfg->n_gen_blocks > 0) {
    ex->gen_w.assign(w->gen, w->gen + cfg->n_gen_blocks); ex->gen_g.assign(grads->gen, grads->gen + cfg->n_gen_blocks);
  }
  ex->proj_in = w->proj_in; ex->proj_out = w->proj_out;
  ex->g_proj_in = (float*)grads->proj_in; ex->g_proj_out = (float*)grads->proj_out;
  ex->mbs.assign(mbs, mbs + cfg->M);
  ex->units.assign(units, units + ex->U);
  ex->enc_slot_of.assign(ex->U, -1); ex->llm_slot_of.assign(cfg->M, -1);
  ex->enc_busy.assign(enc_slots, 0); ex->llm_busy.assign(llm_slots, 0);

  Arena a(arena);
  auto al = [](size_t v) { return align_up(v, 256); };
  ex->scratch = a.take<char>(z.scratch);
  ex->ping[0] = a.take<char>(z.ping); ex->ping[1] = a.take<char>(z.ping);
  const size_t es = ex->es;
  if (cfg->n_gen_blocks > 0) {
    GenSet& g = ex->gen;
    const int maxS = z.maxS_enc;
    for (int i = 0; i < cfg->n_gen_blocks; ++i) {
      g.saved.push_back(a.take<char>(al(saved_bytes(cfg->gen, z.maxT_gen, maxS, cfg->gen_tokens_per_image))));
      g.act.push_back(a.take<char>(al((size_t)z.maxT_gen * cfg->gen.hidden * es)));
      g.dcond.push_back(a.take<char>(al((size_t)maxS * cfg->gen.hidden * es)));
    }
    g.cond = a.take<char>(al((size_t)maxS * cfg->gen.hidden * es));
    g.hsel = a.take<char>(al((size_t)maxS * cfg->llm.hidden * es));
    g.dhsel = a.take<char>(al((size_t)maxS * cfg->llm.hidden * es));
    g.dout = a.take<char>(al((size_t)z.maxT_gen * cfg->gen.hidden * es));
  }
  ex->enc_slots.resize(enc_slots);
  for (auto& s : ex->enc_slots) {
    for (int i = 0; i < cfg->n_enc_blocks; ++i) {
      s.saved.push_back(a.take<char>(al(saved_bytes(cfg->enc, z.maxT_enc, z.maxS_enc, z.maxT_enc))));
      s.act.push_back(a.take<char>(al((size_t)z.maxT_enc * cfg->enc.hidden * es)));
    }
    s.feat = a.take<char>(al((size_t)z.maxT_enc * cfg->llm.hidden * es));
    s.dfeat = a.take<char>(al((size_t)z.maxT_enc * cfg->llm.hidden * es));
  }
  ex->llm_slots.resize(llm_slots);
  for (auto& s : ex->llm_slots) {
    s.x_in = a.take<char>(al((size_t)z.maxT_llm * cfg->llm.hidden * es));
    for (int i = 0; i < cfg->n_llm_blocks; ++i) {
      s.saved.push_back(a.take<char>(al(saved_bytes(cfg->llm, z.maxT_llm, z.maxS_llm, z.maxT_llm))));
      s.act.push_back(a.take<char>(al((size_t)z.maxT_llm * cfg->llm.hidden * es)));
    }
    s.dh_out = cfg->n_gen_blocks > 0 ? a.take<char>(al((size_t)z.maxT_llm * cfg->llm.hidden * es)) : nullptr;
  }
  *out = ex;
  return BM_OK;
}

extern "C" bm_status bm_executor_load_schedule(bm_executor* ex, const int32_t* ops, int32_t n_ops) {
  BM_ARG_CHECK(ex && ops && n_ops > 0, "executor: NULL executor or empty schedule");
  BM_RETURN_IF(bm_check_schedule(ops, n_ops, ex->cfg.M, ex->cfg.unit_size, ex->has_gen() ? 1 : 0, nullptr));
  ex->ops.assign(ops, ops + 2 * (size_t)n_ops);
  return BM_OK;
}

namespace {

// runs the loaded op stream; with `after_op` it is called once before the first op
// (index -1) and once after every op
template <typename F>
bm_status run_ops(bm_executor* ex, float* loss, hipStream_t st, F&& after_op) {
  ex->live = ex->peak = ex->live_enc = ex->peak_enc = 0;
  std::fill(ex->enc_slot_of.begin(), ex->enc_slot_of.end(), -1);
  std::fill(ex->llm_slot_of.begin(), ex->llm_slot_of.end(), -1);
  std::fill(ex->enc_busy.begin(), ex->enc_busy.end(), 0);
  std::fill(ex->llm_busy.begin(), ex->llm_busy.end(), 0);
  BM_RETURN_IF(after_op(-1));
  for (size_t i = 0; i < ex->ops.size() / 2; ++i) {
    const int code = ex->ops[2 * i], idx = ex->ops[2 * i + 1];
    bm_status rc = BM_OK;
    switch (code) {
      case BM_OP_ENC_FWD: rc = enc_fwd(ex, idx, st); break;
      case BM_OP_ENC_BWD: rc = enc_bwd(ex, idx, st); break;
      case BM_OP_LLM_FWD: rc = llm_fwd(ex, idx, st); break;
      case BM_OP_LLM_BWD: rc = llm_bwd(ex, idx, loss, st); break;
      case BM_OP_GEN_FWD: rc = gen_fwd(ex, idx, loss, st); break;
      case BM_OP_GEN_BWD: rc = gen_bwd(ex, idx, st); break;
      default: set_error("executor: opcode %d", code); rc = BM_ERR_INVALID_ARG;
    }
    if (rc != BM_OK) return rc;
    BM_RETURN_IF(after_op((int)i));
  }
  return BM_OK;
}

}  // namespace

extern "C" bm_status bm_executor_execute(bm_executor* ex, float* loss, void* hip_stream) {
  BM_ARG_CHECK(ex && loss, "executor: NULL executor or loss buffer");
  BM_ARG_CHECK(!ex->ops.empty(), "executor: no schedule loaded");
  return run_ops(ex, loss, (hipStream_t)hip_stream, [](int) { return BM_OK; });
}

extern "C" bm_status bm_executor_execute_timed(bm_executor* ex, float* loss, double* op_ms,
                                               double* live_bytes, void* hip_stream) {
  BM_ARG_CHECK(ex && loss && op_ms, "executor: NULL executor, loss buffer or op_ms");
  BM_ARG_CHECK(!ex->ops.empty(), "executor: no schedule loaded");
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t n = ex->ops.size() / 2;
  std::vector<hipEvent_t> ev(n + 1, nullptr);
  bm_status rc = BM_OK;
  for (size_t i = 0; i <= n && rc == BM_OK; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) { set_error("executor: hipEventCreate failed"); rc = BM_ERR_HIP; }
  if (rc == BM_OK)
    rc = run_ops(ex, loss, st, [&](int i) {
      if (hipEventRecord(ev[i + 1], st) != hipSuccess) { set_error("executor: hipEventRecord failed"); return BM_ERR_HIP; }
      if (live_bytes && i >= 0) live_bytes[i] = (double)ex->live;
      return BM_OK;
    });
  if (rc == BM_OK && hipEventSynchronize(ev[n]) != hipSuccess) { set_error("executor: hipEventSynchronize failed"); rc = BM_ERR_HIP; }
  for (size_t i = 0; i < n && rc == BM_OK; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) { set_error("executor: hipEventElapsedTime failed"); rc = BM_ERR_HIP; }
    op_ms[i] = ms;
  }
  for (hipEvent_t e : ev) if (e) (void)hipEventDestroy(e);
  return rc;
}

extern "C" size_t bm_executor_peak_activation_bytes(const bm_executor* ex) { return ex ? ex->peak : 0; }
extern "C" size_t bm_executor_peak_encoder_bytes(const bm_executor* ex) { return ex ? ex->peak_enc : 0; }
extern "C" void bm_executor_destroy(bm_executor* ex) { delete ex; }
