// Variable-length flash attention on the gfx950 matrix cores (bf16 in, fp32
// accumulate, online softmax in base 2), forward and backward.
//
// Packing: a workgroup owns one 128-row tile of ONE sequence and one head, so
// attention is block-diagonal by construction; tiles are enumerated by walking
// cu_seqlens (no padded grid), longest-running tiles first.
//
// Layout trick.  All score matrices are produced TRANSPOSED by the MFMA
// (keys x queries for forward/dQ, queries x keys for dK/dV), so that the
// softmax statistic of a row lives in ONE lane (two lanes for the two 32-lane
// halves) instead of being spread over a wavefront, and the fp32 accumulator
// of one MFMA is -- after conversion to bf16 -- exactly the B operand of the
// next MFMA (P feeds P*V, dS feeds dS*K / dS*Q): probabilities never touch LDS.
// The matching A operands (V^T, K^T, Q^T, dO^T) come from the LDS transpose
// read (ds_read_b64_tr_b16) of tiles stored in their natural [row][dh] form.
// Tiles are XOR-swizzled with a pattern that is conflict-free for both the
// 16-byte row reads and the transpose reads.
//
// Backward is split in two kernels (dK/dV per key tile, dQ per query tile),
// each recomputing P from the saved log-sum-exp: every output element has one
// owner, so there are no floating-point atomics and results are reproducible.
#include "common.h"

#include <type_traits>

namespace bm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Head sizes: 64 and 128 fit the 32x32x16 MFMA exactly; 72 (the DiT blocks) is run
// with its contraction padded to 80 and its output rows padded to 96 by zero chunks
// that exist only in LDS and registers, never in HBM.
template <int DH>
struct HeadDim {
  static constexpr int KS = (DH + 15) / 16;    // k=16 steps when dh is the contraction index
  static constexpr int NB = (DH + 31) / 32;    // 32-row blocks when dh is an output index
  static constexpr int DHL = NB * 32;          // LDS row width in elements
  static constexpr int VCH = DH / 8;           // 16-byte chunks of a row that hold data
};

// ---- swizzled [rows][DHL] bf16 tile -----------------------------------------
template <int DHL>
__device__ inline int tile_swizzle(int row) {      // chunk c of a row sits in slot c ^ tile_swizzle(row)
  if (DHL == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  if (DHL == 96) return (row >> 2) & 3;
  const int v = row >> 1;
  return ((v & 1) << 2) | ((v >> 1) & 3);
}
template <int DHL>
__device__ inline int tile_off(int row, int c) {   // element offset of 16-byte chunk c of a row
  return row * DHL + ((c ^ tile_swizzle<DHL>(row)) << 3);
}

// 8 consecutive dh values (chunk c) of a global row as an MFMA operand; zeros past dh
template <int DH>
__device__ inline bf16x8 load_chunk(const bf16_t* row, int c) {
  if (DH % 16 == 0 || c < HeadDim<DH>::VCH) return *reinterpret_cast<const bf16x8*>(row + c * 8);
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.f;
  return z;
}

// operand fragment, rows of the tile are the MFMA row/col index, dh is the k index:
// lane l -> tile row row0 + l%32, dh = ks*16 + (l/32)*8 .. +7
template <int DH>
__device__ inline bf16x8 frag_rows(const bf16_t* t, int row0, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(t + tile_off<DH>(row0 + (lane & 31), ks * 2 + (lane >> 5)));
}

// A operand X^T: MFMA row = dh index col0 + l%32, k index = tile rows, in the
// order the fp32 accumulator of a transposed score block hands them over:
// half h = l/32 supplies tile rows r0+4h..+3 and r0+8+4h..+3.
template <int DH>
__device__ inline bf16x8 frag_cols(const bf16_t* t, int col0, int r0, int lane) {
  const int gi = lane >> 4, s = lane & 15;
  const int col = col0 + (gi & 1) * 16 + (s & 3) * 4;
  const int row = r0 + (gi >> 1) * 4 + (s >> 2);
  const bf16_t* p0 = t + tile_off<DH>(row, col >> 3) + (col & 7);
  const bf16_t* p1 = t + tile_off<DH>(row + 8, col >> 3) + (col & 7);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p1);
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

// max / sum of a value with the one held by the lane 32 away (the two halves of a wavefront own
// the same score column): v_permlane32_swap exchanges the halves in the vector unit, without the
// trip through the LDS crossbar that a lane shuffle takes
__device__ inline float max_with_other_half(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float sum_with_other_half(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// accumulator rows 8t..8t+7 of a 32x32 block -> bf16 B operand of a k=16 step
__device__ inline bf16x8 acc_to_operand(const f32x16& a, int t) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)a[t * 8 + e];
  return r;
}

// ---- global -> LDS: a [ROWS][DH] tile brought in by NT threads -------------------
// 16-byte loads that write LDS directly (no registers, no LDS store
// instructions): lane l of a wavefront fills bytes [16 l, 16 l + 16) of a 1 KiB run of slots, so the
// swizzle is applied on the global side -- the lane that owns slot s of a row fetches chunk
// s ^ tile_swizzle(row).  Padding slots (head sizes that are no multiple of 32) are never written
// by a load: zero() clears them once.  The loads are asynchronous: wait for vmcnt(0), then a
// workgroup barrier, before any wavefront reads the tile.
template <int ROWS, int DH, int NT>
struct TileAsync {
  static constexpr int DHL = HeadDim<DH>::DHL;
  static constexpr int CPR = DHL / 8;
  static constexpr int SLOTS = ROWS * CPR;
  static constexpr int CH = (SLOTS + NT - 1) / NT;    // loads per thread (the last round may be short)
  // UNI: every load of a thread has the same chunk, and rows a fixed distance apart
  static constexpr bool UNI = NT % CPR == 0 && (NT / CPR) % 16 == 0 && SLOTS % NT == 0;
  static constexpr int RSTEP = NT / CPR, NV = UNI ? 1 : CH;
  static_assert(SLOTS % 64 == 0 && NT % 64 == 0, "a tile is a whole number of 1 KiB runs");
  static constexpr bool ALL_LIVE = DHL == DH && SLOTS % NT == 0;   // no padding slot, no short round
  uint32_t goff[NV];    // byte offset of a load from the tile's first row (full tiles)
  int tid_;             // the thread's index among the NT that bring the tile in
  // (row, chunk) of load i; false: it would fill a padding slot or lies past the tile
  __device__ inline bool place(int i, int* row, int* chunk, int tid) const {
    const int id = tid + i * NT;
    *row = id / CPR;
    *chunk = (id % CPR) ^ tile_swizzle<DHL>(*row);
    return ALL_LIVE || (id < SLOTS && *chunk < HeadDim<DH>::VCH);
  }
  __device__ inline void init(int ld, int tid) {
    tid_ = tid;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int row, c;
      place(i, &row, &c, tid);
      goff[i] = (uint32_t)row * (uint32_t)ld * 2u + (uint32_t)c * 16u;
    }
  }
  // One 16-byte load per lane straight into LDS.  Written as inline assembly so that the compiler does
  // not see an LDS write in flight: it would otherwise make every LDS read that follows wait for
  // vmcnt(0) and the tile would no longer stream in behind the arithmetic.  The caller orders the
  // reads of a tile after wait_async_tiles() and a barrier.
  static __device__ inline void load16(const void* base, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
  }
  // base: first row of the tile (wave-uniform); rows_left: valid rows from there (>= 1), rows beyond
  // them are clamped to the last valid one (their results are masked or unused); wave: wave-uniform
  __device__ inline void issue(const bf16_t* __restrict__ base_in, int ld, int rows_left, bf16_t* t,
                               int wave) const {
    // the base goes into the asm statement as a scalar register pair: say so, wherever the caller's
    // arithmetic left it
    const uint64_t b64 = reinterpret_cast<uint64_t>(base_in);
    const bf16_t* base = reinterpret_cast<const bf16_t*>(
        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b64 >> 32)) << 32) |
        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b64));
    rows_left = __builtin_amdgcn_readfirstlane(rows_left);
    const uint32_t dst = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)(t + wave * 512);
    if (rows_left >= ROWS) {
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        int row, c;
        // (UNI: the distance between a thread's loads goes into the scalar base, not into a register each)
        if (place(i, &row, &c, tid_))
          load16(base + (UNI ? (size_t)(i * RSTEP) * ld : (size_t)0), goff[UNI ? 0 : i], dst + i * NT * 16);
      }
    } else {
      // a cut tile (the last one of a sequence): offsets from scratch, rows clamped.  The thread index
      // passes through an empty asm so that none of this is computed ahead of the loop and kept in
      // registers for the one step that needs it.
      int t_op = tid_;
      asm volatile("" : "+v"(t_op));
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        int row, c;
        if (place(i, &row, &c, t_op))
          load16(base, (uint32_t)min(row, rows_left - 1) * (uint32_t)ld * 2u + (uint32_t)c * 16u, dst + i * NT * 16);
      }
    }
  }
  static __device__ inline void zero_padding(bf16_t* t, int tid) {
    if (DHL == DH) return;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int id = tid + i * NT;
      const int r = id / CPR, c = (id % CPR) ^ tile_swizzle<DHL>(r);
      if (id < SLOTS && c >= HeadDim<DH>::VCH) *reinterpret_cast<u32x4*>(t + id * 8) = u32x4{0u, 0u, 0u, 0u};
    }
  }
};
// The tile loads are invisible to the compiler's wait-count bookkeeping, so the wait for them is
// written out as well.  A vmcnt wait that the compiler adds for one of ITS loads would also wait for
// tile loads in flight: settle_compiler_loads() (a wait the bookkeeping does read) goes once in front
// of a loop that streams tiles, after the kernel's ordinary loads, so that none is added inside.
__device__ inline void wait_async_tiles() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ inline void settle_compiler_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */ }

// The order in which the tiles of the sequences are handed out: workgroups are dispatched in id
// order, so the sequences whose tiles run longest go first and the short ones fill the tail of the
// launch.  Built on the host from the host copy of the offsets (the same copy that sizes the grid)
// and passed by value in the kernel arguments: nothing to allocate or copy, and a workgroup finds
// its tile from one batch of scalar loads instead of a dependent load per sequence.  Any order
// gives the same results, only the schedule changes.  n == 0: no table (more than 64 sequences),
// the kernel walks the offsets in pack order.
struct SeqOrder {
  int n;                // positions in use, a multiple of 16
  uint32_t w[64];       // position i: sequence index in bits 0..7, its number of tiles above
};

// cu_tiles: offsets of the side that is cut into tiles of `rows` rows; cu_cost: offsets of the side
// a tile loops over (its running time).  sorted = false keeps the pack order: under a causal mask
// a pack has tiles of every length whatever the order, and the long sequences' tiles all running at
// once measured slower (their operands no longer fit the L2 of an XCD together).
SeqOrder make_seq_order(const int32_t* cu_tiles, const int32_t* cu_cost, int S, int rows, bool sorted) {
  SeqOrder o;
  o.n = 0;
  for (int i = 0; i < 64; ++i) o.w[i] = 0;          // unused positions: sequence 0, no tile
  if (S < 1 || S > 64) return o;
  for (int s = 0; s < S; ++s)
    if ((cu_tiles[s + 1] - cu_tiles[s] + rows - 1) / rows >= (1 << 24)) return o;
  unsigned char idx[64];
  for (int i = 0; i < S; ++i) idx[i] = (unsigned char)i;
  // stable insertion sort by descending length
  for (int i = 1; sorted && i < S; ++i) {
    const unsigned char x = idx[i];
    const int lx = cu_cost[x + 1] - cu_cost[x];
    int j = i;
    while (j > 0 && cu_cost[idx[j - 1] + 1] - cu_cost[idx[j - 1]] < lx) { idx[j] = idx[j - 1]; --j; }
    idx[j] = x;
  }
  o.n = (S + 15) / 16 * 16;
  for (int i = 0; i < S; ++i) {
    const int nt = (cu_tiles[idx[i] + 1] - cu_tiles[idx[i]] + rows - 1) / rows;
    o.w[i] = ((uint32_t)nt << 8) | idx[i];
  }
  return o;
}

// which (sequence, tile) a linear tile id is; tiles of `rows` rows, later tiles of a
// sequence first (under a causal mask they are the long ones).  Wave-uniform throughout.
__device__ inline bool find_tile(const int32_t* __restrict__ cu, const SeqOrder& ord, int S, int rows, int id,
                                 int* seq, int* tile, int* ntiles) {
  if (ord.n == 0) {
    for (int s = 0; s < S; ++s) {
      const int L = cu[s + 1] - cu[s];
      const int nt = (L + rows - 1) / rows;
      if (id < nt) { *seq = s; *tile = nt - 1 - id; *ntiles = nt; return true; }
      id -= nt;
    }
    return false;
  }
  for (int s0 = 0; s0 < ord.n; s0 += 16) {
    uint32_t e[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) e[j] = ord.w[s0 + j];
    int found = -1, fid = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {               // branch-free choice among the sixteen
      const int n = (int)(e[j] >> 8);
      const bool here = found < 0 && id < n;
      found = here ? (int)e[j] : found;
      fid = here ? id : fid;
      id -= found < 0 ? n : 0;
    }
    if (found >= 0) {
      const int nt = found >> 8;
      *seq = found & 255; *tile = nt - 1 - fid; *ntiles = nt;
      return true;
    }
  }
  return false;
}

// Linear workgroup id -> (tile id, head).  Heads vary fastest, and since workgroup
// ids go round-robin over the 8 XCDs, head index i lands on XCD i%8: give XCD x
// the consecutive heads x*(H/8).., so every tile of one head -- and the q heads of
// one GQA group -- meet their K/V in the same XCD's L2.
__device__ inline void tile_and_head(int H, int* tile, int* head) {
  const int b = blockIdx.x;
  const int i = b % H;
  *tile = b / H;
  *head = (H % 8 == 0) ? (i % 8) * (H / 8) + i / 8 : i;
}

// =============================================================================
// forward
// =============================================================================
constexpr int FQ = 128;   // query rows per workgroup (32 per wavefront)
constexpr int FK = 64;    // keys per step

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void fa_fwd_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int ld,
    int ldk, const int32_t* __restrict__ cu, const int32_t* __restrict__ cuk, int S,
    bf16_t* __restrict__ o, int ldo, float* __restrict__ lse, int Ttot, int Hq, int group,
    float scale_log2, SeqOrder ord) {
  // K and V tiles are double-buffered: tile kt+1 streams into LDS while tile kt is consumed
  constexpr int TILE = FK * HeadDim<DH>::DHL;
  __shared__ __attribute__((aligned(1024))) bf16_t Kbuf[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vbuf[2 * TILE];
  int seq, qt, nqt, tile_id, hq;
  tile_and_head(Hq, &tile_id, &hq);
  if (!find_tile(cu, ord, S, FQ, tile_id, &seq, &qt, &nqt)) return;
  const int hk = hq / group;
  const int lo = cu[seq], L = cu[seq + 1] - lo;
  // keys and values may be packed on their own (a chunk of a context-parallel partition)
  const int lok = cuk[seq], Lk = cuk[seq + 1] - lok;
  const int q0 = qt * FQ;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5;
  const int qpos = q0 + wave * 32 + (lane & 31);          // this lane's query (column of S^T)
  const int qrow = min(qpos, L - 1);
  if (Lk == 0) {
    // no key in this chunk (workgroup-uniform): zero output, lse = -inf
    if (qpos < L) {
      bf16_t* op = o + (size_t)(lo + qpos) * ldo + hq * DH;
      for (int c = half * (DH / 2); c < (half + 1) * (DH / 2); c += 4) {
        bf16x4 z = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
        *reinterpret_cast<bf16x4*>(op + c) = z;
      }
      if (half == 0) lse[(size_t)hq * Ttot + lo + qpos] = -INFINITY;
    }
    return;
  }

  bf16x8 qf[HeadDim<DH>::KS];
  {
    const bf16_t* qp = q + (size_t)(lo + qrow) * ld + hq * DH;
#pragma unroll
    for (int ks = 0; ks < HeadDim<DH>::KS; ++ks) qf[ks] = load_chunk<DH>(qp, ks * 2 + half);
  }
  f32x16 oacc[HeadDim<DH>::NB];
#pragma unroll
  for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[j][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  const int kend = CAUSAL ? min(Lk, q0 + FQ) : Lk;
  const int nkt = (kend + FK - 1) / FK;
  const bf16_t* kbase = k + (size_t)lok * ldk + hk * DH;
  const bf16_t* vbase = v + (size_t)lok * ldk + hk * DH;
  using Tile = TileAsync<FK, DH, 256>;
  Tile tile;
  tile.init(ldk, tid);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    Tile::zero_padding(Kbuf + b * TILE, tid);
    Tile::zero_padding(Vbuf + b * TILE, tid);
  }
  tile.issue(kbase, ldk, Lk, Kbuf, wave_u);
  tile.issue(vbase, ldk, Lk, Vbuf, wave_u);
  settle_compiler_loads();                 // the Q fragments (and, with them, tile 0)

  // The step comes in two copies, without and with the per-element mask test, each in a loop of
  // its own: the leading key tiles lie wholly inside the sequence (and before the diagonal under a
  // causal mask) and need no test; written as a run-time condition inside the unrolled code, the
  // test becomes compare/select pairs that every step pays for.  Every wavefront runs nkt steps
  // in total (the split may differ between wavefronts; the barrier count per step does not).
  auto step = [&](int kt, auto masked, auto parity) {
    constexpr bool MASKED = decltype(masked)::value;
    constexpr int PAR = decltype(parity)::value;
    const bf16_t* Ks = Kbuf + PAR * TILE;
    const bf16_t* Vs = Vbuf + PAR * TILE;
    // one barrier per step: tile kt has landed for every wavefront, and every wavefront is done
    // with tile kt-1, whose buffer the loads of tile kt+1 overwrite
    wait_async_tiles();
    __syncthreads();
    if (kt + 1 < nkt) {
      const size_t next = (size_t)(kt + 1) * FK * ldk;
      tile.issue(kbase + next, ldk, Lk - (kt + 1) * FK, Kbuf + (1 - PAR) * TILE, wave_u);
      tile.issue(vbase + next, ldk, Lk - (kt + 1) * FK, Vbuf + (1 - PAR) * TILE, wave_u);
    }
    const int key0 = kt * FK;
    // S^T = K Q^T for both 32-key blocks first: the MFMAs of block 1 run while the
    // softmax arithmetic of block 0 occupies the vector unit, and the P V MFMAs of
    // block 0 run under the softmax of block 1.
    f32x16 sacc[FK / 32];
#pragma unroll
    for (int b = 0; b < FK / 32; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
    {
      // K fragments are requested from LDS AHEAD MFMAs before their use (a ring of register sets)
      constexpr int KS = HeadDim<DH>::KS, NSTEP = (FK / 32) * KS, AHEAD = 2;
      bf16x8 fk[AHEAD + 1];
#pragma unroll
      for (int n = 0; n < AHEAD && n < NSTEP; ++n) fk[n] = frag_rows<HeadDim<DH>::DHL>(Ks, (n / KS) * 32, n % KS, lane);
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) {
        const int m = n + AHEAD;
        if (m < NSTEP) fk[m % (AHEAD + 1)] = frag_rows<HeadDim<DH>::DHL>(Ks, (m / KS) * 32, m % KS, lane);
        sacc[n / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[n % (AHEAD + 1)], qf[n % KS], sacc[n / KS], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // mask: keys past the sequence end, and keys after the query under a causal mask
#pragma unroll
    for (int b = 0; b < FK / 32; ++b) {
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (MASKED) {
          const int key = key0 + b * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (key >= Lk || (CAUSAL && key > qpos)) sacc[b][r] = -INFINITY;
        }
        mx = fmaxf(mx, sacc[b][r]);
      }
      mx = max_with_other_half(mx) * scale_log2;
      // Lazy rescaling: the running maximum only moves (and O, l are only rescaled)
      // when some row's maximum grew by more than 2^8; until then probabilities are
      // taken relative to the older maximum (they stay below 2^8, exact in fp32).
      if (__builtin_amdgcn_ballot_w64(mx > m + 8.0f) != 0) {
        const float m_new = fmaxf(m, mx);
        const float corr = __builtin_amdgcn_exp2f(m - m_new);   // m = -inf at the start: 0
        m = m_new;
        lsum *= corr;
#pragma unroll
        for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[j][r] *= corr;
      }
      float psum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[b][r], scale_log2, -m));   // masked: exp2(-inf) = 0
        sacc[b][r] = p;
        psum += p;
      }
      lsum += psum;
      const bf16x8 p0 = acc_to_operand(sacc[b], 0), p1 = acc_to_operand(sacc[b], 1);
      // O^T += V^T P^T, the transposed V operands requested one pair of MFMAs ahead
      {
        constexpr int NB = HeadDim<DH>::NB;
        bf16x8 fr[2][2];
        fr[0][0] = frag_cols<HeadDim<DH>::DHL>(Vs, 0, b * 32, lane);
        fr[0][1] = frag_cols<HeadDim<DH>::DHL>(Vs, 0, b * 32 + 16, lane);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          if (j + 1 < NB) {
            fr[(j + 1) & 1][0] = frag_cols<HeadDim<DH>::DHL>(Vs, (j + 1) * 32, b * 32, lane);
            fr[(j + 1) & 1][1] = frag_cols<HeadDim<DH>::DHL>(Vs, (j + 1) * 32, b * 32 + 16, lane);
          }
          oacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][0], p0, oacc[j], 0, 0, 0);
          oacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][1], p1, oacc[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  // tiles kt < n_plain need no test: key0 + FK <= Lk, and key0 + FK - 1 <= this wavefront's first query
  int n_plain = Lk / FK;
  if (CAUSAL) n_plain = min(n_plain, (q0 + wave * 32 + 1) / FK);
  n_plain = min(n_plain, nkt);
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  for (int kt = 0; kt < nkt; ++kt) {
    const bool plain = kt < n_plain;
    if (kt & 1) { if (plain) step(kt, std::false_type{}, P1{}); else step(kt, std::true_type{}, P1{}); }
    else { if (plain) step(kt, std::false_type{}, P0{}); else step(kt, std::true_type{}, P0{}); }
  }
  lsum = sum_with_other_half(lsum);
  if (qpos < L) {
    const float inv = 1.0f / lsum;
    bf16_t* op = o + (size_t)(lo + qpos) * ldo + hq * DH;
#pragma unroll
    for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(oacc[j][g * 4 + e] * inv);
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH)
          *reinterpret_cast<bf16x4*>(op + j * 32 + g * 8 + half * 4) = w;
      }
    if (half == 0) lse[(size_t)hq * Ttot + lo + qpos] = (m + log2f(lsum)) * LN2;
  }
}

int count_tiles(const int32_t* cu_host, int S, int rows) {
  long n = 0;
  for (int s = 0; s < S; ++s) n += (cu_host[s + 1] - cu_host[s] + rows - 1) / rows;
  return (int)n;
}

template <int DH>
bm_status fwd_launch(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
  dim3 grid(count_tiles(a.cu_host, a.S, FQ) * a.Hq), block(256);
  if (grid.x == 0) return BM_OK;
  const float sl2 = LOG2E / sqrtf((float)a.dh);
  // a query tile runs as long as its sequence has keys
  const SeqOrder ord = make_seq_order(a.cu_host, a.kv_cu_host(), a.S, FQ, !a.causal);
#define BM_L(C)                                                                                  \
  hipLaunchKernelGGL((fa_fwd_kernel<DH, C>), grid, block, 0, st, (const bf16_t*)a.q,             \
                     (const bf16_t*)a.k, (const bf16_t*)a.v, a.ld_qkv, a.kv_ld(), a.cu_dev,      \
                     a.kv_cu_dev(), a.S, (bf16_t*)o, a.Hq * a.dh, lse, a.T, a.Hq, a.Hq / a.Hkv, sl2, ord)
  if (a.causal) BM_L(true); else BM_L(false);
#undef BM_L
  BM_CHECK_LAUNCH("fa_fwd");
  return BM_OK;
}

// =============================================================================
// backward
// =============================================================================
// delta[h, t] = sum_c dO[t,h,c] * O[t,h,c]; 8 (head size 64) or 16 lanes share one (row, head),
// 16 bytes each, so a wavefront reads whole contiguous row segments
template <int DH> struct DeltaLanes { static constexpr int N = DH <= 64 ? 8 : 16, SHIFT = DH <= 64 ? 3 : 4; };
template <int DH>
__global__ void fa_delta_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o, int ldo,
                                float* __restrict__ delta, int Ttot, int Hq) {
  constexpr int LP = DeltaLanes<DH>::N;
  const long gid = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> DeltaLanes<DH>::SHIFT;
  const int c = (threadIdx.x & (LP - 1)) * 8;
  float s = 0.f;
  const bool live = gid < (long)Ttot * Hq;
  const int t = live ? (int)(gid / Hq) : 0, hq = live ? (int)(gid % Hq) : 0;
  if (live && c < DH) {
    float a[8], b[8];
    load16(o + (size_t)t * ldo + hq * DH + c, a);
    load16(d_o + (size_t)t * ldo + hq * DH + c, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) s = fmaf(a[e], b[e], s);
  }
#pragma unroll
  for (int off = LP / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (live && c == 0) delta[(size_t)hq * Ttot + t] = s;
}

constexpr int BK_KEYS = 128;   // keys per workgroup in the dK/dV kernel (32 per wavefront)
constexpr int BK_Q = 64;       // query rows per step

// dK, dV of one 128-key tile of one kv head: walks the q heads of the group and the
// query tiles; scores are kept as S[q, key] so that P and dS are B operands as they are.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256, DH <= 64 ? 2 : 1) void fa_bwd_dkdv_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int ld,
    int ldk, const bf16_t* __restrict__ d_o, int ldo, const float* __restrict__ lse,
    const float* __restrict__ delta, const int32_t* __restrict__ cuq, const int32_t* __restrict__ cu,
    int S, bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int ldd, int Tq, int Ttot, int Hkv, int group,
    float scale, float scale_log2, int gsplit,
    float* __restrict__ part /* [gsplit][2][Ttot][Hkv*DH] fp32 when gsplit > 1 */, SeqOrder ord) {
  // cu, Ttot, ldk: the packing of the keys/values (and of dk, dv); cuq, Tq, ld: of the queries
  // Q and dO tiles are double-buffered and streamed into LDS (see TileAsync)
  constexpr int TILE = BK_Q * HeadDim<DH>::DHL;
  __shared__ __attribute__((aligned(1024))) bf16_t Qbuf[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Dbuf[2 * TILE];
  __shared__ __attribute__((aligned(16))) float Lbuf[2 * BK_Q];
  __shared__ __attribute__((aligned(16))) float Dlbuf[2 * BK_Q];
  int seq, kt, nkt, tile_id, hk;
  // with gsplit > 1 a workgroup takes group/gsplit of the q heads that share this kv head
  // and leaves an fp32 partial; the (kv head, q-head part) pair plays the head's role
  int hk_gs;
  tile_and_head(Hkv * gsplit, &tile_id, &hk_gs);
  hk = hk_gs / gsplit;
  const int gs = hk_gs % gsplit;
  const int gpart = group / gsplit;
  if (!find_tile(cu, ord, S, BK_KEYS, tile_id, &seq, &kt, &nkt)) return;
  kt = nkt - 1 - kt;                                   // early key tiles see the most queries
  const int lo = cu[seq], L = cu[seq + 1] - lo;
  const int loq = cuq[seq], Lq = cuq[seq + 1] - loq;
  const int kb0 = kt * BK_KEYS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int kpos = kb0 + wave * 32 + (lane & 31);       // this lane's key (column of S)
  const int krow = min(kpos, L - 1);

  bf16x8 kf[HeadDim<DH>::KS], vf[HeadDim<DH>::KS];
  {
    const bf16_t* kp = k + (size_t)(lo + krow) * ldk + hk * DH;
    const bf16_t* vp = v + (size_t)(lo + krow) * ldk + hk * DH;
#pragma unroll
    for (int ks = 0; ks < HeadDim<DH>::KS; ++ks) {
      kf[ks] = load_chunk<DH>(kp, ks * 2 + half);
      vf[ks] = load_chunk<DH>(vp, ks * 2 + half);
    }
  }
  f32x16 dkacc[HeadDim<DH>::NB], dvacc[HeadDim<DH>::NB];
#pragma unroll
  for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[j][r] = 0.f; dvacc[j][r] = 0.f; }

  const int qstart = CAUSAL ? (kb0 / BK_Q) * BK_Q : 0;
  const int nqt = Lq > qstart ? (Lq - qstart + BK_Q - 1) / BK_Q : 0;   // no query: dk = dv = 0
  const int iters = nqt * gpart;
  using Tile = TileAsync<BK_Q, DH, 256>;
  Tile tq, td;
  tq.init(ld, tid);
  td.init(ldo, tid);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  float st_l = 0.f, st_d = 0.f;
  auto fetch = [&](int it, int par) {
    const int hq = hk * group + gs * gpart + it / nqt;
    const int q0 = qstart + (it % nqt) * BK_Q;
    tq.issue(q + ((size_t)loq + q0) * ld + hq * DH, ld, Lq - q0, Qbuf + par * TILE, wave_u);
    td.issue(d_o + ((size_t)loq + q0) * ldo + hq * DH, ldo, Lq - q0, Dbuf + par * TILE, wave_u);
    if (tid < BK_Q) {
      const int qi = min(q0 + tid, Lq - 1);
      st_l = lse[(size_t)hq * Tq + loq + qi];      // used (and waited for) when the next step opens
      st_d = delta[(size_t)hq * Tq + loq + qi];
    }
  };
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    Tile::zero_padding(Qbuf + b * TILE, tid);
    Tile::zero_padding(Dbuf + b * TILE, tid);
  }
  if (iters > 0) fetch(0, 0);
  settle_compiler_loads();                              // K and V fragments, lse, delta (and, with them, tile 0)
  // one step; MASKED is a compile-time copy with the per-element tests (see the forward kernel)
  constexpr bool FOLD_DELTA = DH <= 64;
  auto step = [&](int it, auto masked, auto parity) {
    constexpr bool MASKED = decltype(masked)::value;
    constexpr int PAR = decltype(parity)::value;
    const bf16_t* Qs = Qbuf + PAR * TILE;
    const bf16_t* Ds = Dbuf + PAR * TILE;
    const float* Ls = Lbuf + PAR * BK_Q;
    const float* Dl = Dlbuf + PAR * BK_Q;
    if (tid < BK_Q) { Lbuf[PAR * BK_Q + tid] = st_l * LOG2E; Dlbuf[PAR * BK_Q + tid] = st_d; }
    wait_async_tiles();
    __syncthreads();      // tile `it` is there for everyone, and everyone is done with tile it-1
    if (it + 1 < iters) fetch(it + 1, 1 - PAR);
    const int q0 = qstart + (it % nqt) * BK_Q;
    // S = Q K^T and dP = dO V^T for both 32-query blocks first, then per block the
    // softmax arithmetic (under the other block's MFMAs) followed by its dV / dK MFMAs.
    f32x16 sacc[BK_Q / 32], dpacc[BK_Q / 32];
#pragma unroll
    for (int qb = 0; qb < BK_Q / 32; ++qb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[qb][r] = 0.f; dpacc[qb][r] = 0.f; }
      // With several resident wavefronts to hide the LDS read, dP starts at -delta of its query
      // row, so that the MFMAs leave dP - delta: one subtraction per score element less on the
      // vector unit.  (With one wavefront per SIMD the read in front of the MFMAs costs more.)
      if (FOLD_DELTA) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(Dl + qb * 32 + g * 8 + half * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) dpacc[qb][g * 4 + e] = -d4[e];
        }
      }
    }
    {
      // the operand fragments of step n + AHEAD are requested from LDS before the MFMAs of step n
      // are issued (a ring of AHEAD + 1 register sets): with one wavefront per SIMD nothing else
      // would cover the LDS latency in front of every MFMA
      constexpr int KS = HeadDim<DH>::KS, NSTEP = (BK_Q / 32) * KS, AHEAD = 2;
      bf16x8 fq[AHEAD + 1], fd[AHEAD + 1];
#pragma unroll
      for (int n = 0; n < AHEAD && n < NSTEP; ++n) {
        fq[n] = frag_rows<HeadDim<DH>::DHL>(Qs, (n / KS) * 32, n % KS, lane);
        fd[n] = frag_rows<HeadDim<DH>::DHL>(Ds, (n / KS) * 32, n % KS, lane);
      }
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) {
        const int qb = n / KS, ks = n % KS, m = n + AHEAD;
        if (m < NSTEP) {
          fq[m % (AHEAD + 1)] = frag_rows<HeadDim<DH>::DHL>(Qs, (m / KS) * 32, m % KS, lane);
          fd[m % (AHEAD + 1)] = frag_rows<HeadDim<DH>::DHL>(Ds, (m / KS) * 32, m % KS, lane);
        }
        sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % (AHEAD + 1)], kf[ks], sacc[qb], 0, 0, 0);
        dpacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[n % (AHEAD + 1)], vf[ks], dpacc[qb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int qb = 0; qb < BK_Q / 32; ++qb) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int qoff = qb * 32 + g * 8 + half * 4;
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(Ls + qoff);
        f32x4 d4 = {0.f, 0.f, 0.f, 0.f};
        if (!FOLD_DELTA) d4 = *reinterpret_cast<const f32x4*>(Dl + qoff);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = g * 4 + e;
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[qb][r], scale_log2, -l4[e]));
          if (MASKED) {
            const int qi = q0 + qoff + e;
            if (qi >= Lq || kpos >= L || (CAUSAL && kpos > qi)) p = 0.f;
          }
          sacc[qb][r] = p;
          dpacc[qb][r] = FOLD_DELTA ? p * dpacc[qb][r] : p * (dpacc[qb][r] - d4[e]);
        }
      }
      const bf16x8 p0 = acc_to_operand(sacc[qb], 0), p1 = acc_to_operand(sacc[qb], 1);
      const bf16x8 s0 = acc_to_operand(dpacc[qb], 0), s1 = acc_to_operand(dpacc[qb], 1);
      {
        // dV += dO^T P, dK += Q^T dS: 4 MFMAs per 32 columns of dh, their transposed operands
        // requested one group ahead
        constexpr int NB = HeadDim<DH>::NB;
        bf16x8 fr[2][4];
        auto request = [&](int j, bf16x8 (&f)[4]) {
          f[0] = frag_cols<HeadDim<DH>::DHL>(Ds, j * 32, qb * 32, lane);
          f[1] = frag_cols<HeadDim<DH>::DHL>(Ds, j * 32, qb * 32 + 16, lane);
          f[2] = frag_cols<HeadDim<DH>::DHL>(Qs, j * 32, qb * 32, lane);
          f[3] = frag_cols<HeadDim<DH>::DHL>(Qs, j * 32, qb * 32 + 16, lane);
        };
        request(0, fr[0]);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          if (j + 1 < NB) request(j + 1, fr[(j + 1) & 1]);
          dvacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][0], p0, dvacc[j], 0, 0, 0);
          dvacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][1], p1, dvacc[j], 0, 0, 0);
          dkacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][2], s0, dkacc[j], 0, 0, 0);
          dkacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][3], s1, dkacc[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  // Which query tiles need the tests: all of them when this key tile is cut by the sequence end;
  // else, per q head, the first ones under a causal mask (queries before this wavefront's last
  // key) and the last one when it is cut by the sequence end.  Every wavefront runs `iters`
  // steps; only the split between the copies differs.
  {
    // (one call site per copy of the step: with two the compiler stops inlining them)
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    const bool all_masked = kb0 + BK_KEYS > L;
    const int n_front = CAUSAL ? min(nqt, (wave * 32 + 32 + BK_Q - 1) / BK_Q) : 0;
    const int n_whole = max(n_front, (Lq - qstart) % BK_Q ? nqt - 1 : nqt);
    for (int it = 0, t = 0; it < iters; ++it, t = (t + 1 == nqt ? 0 : t + 1)) {
      const bool masked = all_masked || t < n_front || t >= n_whole;
      if (it & 1) { if (masked) step(it, std::true_type{}, P1{}); else step(it, std::false_type{}, P1{}); }
      else { if (masked) step(it, std::true_type{}, P0{}); else step(it, std::false_type{}, P0{}); }
    }
  }
  if (kpos < L && gsplit > 1) {
    const size_t plane = (size_t)Ttot * Hkv * DH;
    float* pk = part + ((size_t)gs * 2 + 0) * plane + (size_t)(lo + kpos) * (Hkv * DH) + hk * DH;
    float* pv = part + ((size_t)gs * 2 + 1) * plane + (size_t)(lo + kpos) * (Hkv * DH) + hk * DH;
#pragma unroll
    for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH) {
          *reinterpret_cast<f32x4*>(pk + j * 32 + g * 8 + half * 4) =
              f32x4{dkacc[j][g * 4] * scale, dkacc[j][g * 4 + 1] * scale, dkacc[j][g * 4 + 2] * scale, dkacc[j][g * 4 + 3] * scale};
          *reinterpret_cast<f32x4*>(pv + j * 32 + g * 8 + half * 4) =
              f32x4{dvacc[j][g * 4], dvacc[j][g * 4 + 1], dvacc[j][g * 4 + 2], dvacc[j][g * 4 + 3]};
        }
  } else if (kpos < L) {
    bf16_t* pk = dk + (size_t)(lo + kpos) * ldd + hk * DH;
    bf16_t* pv = dv + (size_t)(lo + kpos) * ldd + hk * DH;
#pragma unroll
    for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 wk, wv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wk[e] = (bf16_t)(dkacc[j][g * 4 + e] * scale);
          wv[e] = (bf16_t)dvacc[j][g * 4 + e];
        }
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH) {
          *reinterpret_cast<bf16x4*>(pk + j * 32 + g * 8 + half * 4) = wk;
          *reinterpret_cast<bf16x4*>(pv + j * 32 + g * 8 + half * 4) = wv;
        }
      }
  }
}

// dK, dV at head sizes above 64, where one wavefront cannot hold both accumulators next to a
// second resident wavefront: every 32-key block of the 128-key tile is shared by a PAIR of
// wavefronts that sit on the same SIMD (wavefronts w and w+4 of the 512-thread workgroup).
//   role 0 ("value" wavefront): S = Q K^T -> P = exp2(S*scale - lse), hands P to its partner
//                               through LDS, dV += dO^T P
//   role 1 ("key" wavefront):   dP = dO V^T, takes P, dS = P (dP - delta), dK += Q^T dS
// Each wavefront keeps one accumulator and one of K / V in registers (about 200 registers), so
// two are resident per SIMD and one's vector work runs under the other's MFMAs.  P travels as
// bf16 in the operand layout: role 0 feeds exactly these values to its own MFMAs, and role 1
// owns the same (key, query) elements in the same lanes, so the exchange is lane-private.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(512, 2) void fa_bwd_dkdv_pair_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int ld,
    int ldk, const bf16_t* __restrict__ d_o, int ldo, const float* __restrict__ lse,
    const float* __restrict__ delta, const int32_t* __restrict__ cuq, const int32_t* __restrict__ cu,
    int S, bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int ldd, int Tq, int Ttot, int Hkv, int group,
    float scale, float scale_log2, int gsplit,
    float* __restrict__ part /* [gsplit][2][Ttot][Hkv*DH] fp32 when gsplit > 1 */, SeqOrder ord) {
  constexpr int DHL = HeadDim<DH>::DHL, KS = HeadDim<DH>::KS, NB = HeadDim<DH>::NB, NQB = BK_Q / 32;
  // Q and dO tiles are double-buffered and streamed into LDS (see TileAsync): with one workgroup
  // per CU nothing else runs while a tile is parked between two barriers
  constexpr int TILE = BK_Q * DHL;
  __shared__ __attribute__((aligned(1024))) bf16_t Qbuf[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Dbuf[2 * TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ps[4 * NQB * 2 * 64 * 8];   // [key block][q block][half k-step][lane] x 16 B
  __shared__ __attribute__((aligned(16))) float Lbuf[2 * BK_Q];
  __shared__ __attribute__((aligned(16))) float Dlbuf[2 * BK_Q];
  int seq, kt, nkt, tile_id, hk, hk_gs;
  tile_and_head(Hkv * gsplit, &tile_id, &hk_gs);
  hk = hk_gs / gsplit;
  const int gs = hk_gs % gsplit;
  const int gpart = group / gsplit;
  if (!find_tile(cu, ord, S, BK_KEYS, tile_id, &seq, &kt, &nkt)) return;
  kt = nkt - 1 - kt;                                   // early key tiles see the most queries
  const int lo = cu[seq], L = cu[seq + 1] - lo;
  const int loq = cuq[seq], Lq = cuq[seq + 1] - loq;
  const int kb0 = kt * BK_KEYS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int kb = wave & 3, role = wave >> 2;            // wavefronts w and w+4 share a SIMD
  const int tid_r = tid & 255;                          // index inside the role's 256 threads
  const int kpos = kb0 + kb * 32 + (lane & 31);         // this lane's key (column of S)
  const int krow = min(kpos, L - 1);

  // role 0 keeps K (for S), role 1 keeps V (for dP)
  bf16x8 kvf[KS];
  {
    const bf16_t* p = (role == 0 ? k : v) + (size_t)(lo + krow) * ldk + hk * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kvf[ks] = load_chunk<DH>(p, ks * 2 + half);
  }
  f32x16 acc[NB];                                       // role 0: dV^T, role 1: dK^T (unscaled)
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

  const int qstart = CAUSAL ? (kb0 / BK_Q) * BK_Q : 0;
  const int nqt = Lq > qstart ? (Lq - qstart + BK_Q - 1) / BK_Q : 0;   // no query: dk = dv = 0
  const int iters = nqt * gpart;
  // role 0's wavefronts bring in the Q tile, role 1's the dO tile; lse and delta of the tile's
  // queries pass through registers of the first wavefront
  using Tile = TileAsync<BK_Q, DH, 256>;
  Tile tile;
  tile.init(role == 0 ? ld : ldo, tid_r);
  const int wave_r = __builtin_amdgcn_readfirstlane(wave & 3);
  const int role_u = __builtin_amdgcn_readfirstlane(role);
  float st_l = 0.f, st_d = 0.f;
  auto fetch = [&](int it, int par) {
    const int hq = hk * group + gs * gpart + it / nqt;
    const int q0 = qstart + (it % nqt) * BK_Q;
    if (role_u == 0) tile.issue(q + ((size_t)loq + q0) * ld + hq * DH, ld, Lq - q0, Qbuf + par * TILE, wave_r);
    else tile.issue(d_o + ((size_t)loq + q0) * ldo + hq * DH, ldo, Lq - q0, Dbuf + par * TILE, wave_r);
    if (tid < BK_Q) {
      const int qi = min(q0 + tid, Lq - 1);
      st_l = lse[(size_t)hq * Tq + loq + qi];     // used (and waited for) when the next step opens
      st_d = delta[(size_t)hq * Tq + loq + qi];
    }
  };
#pragma unroll
  for (int b = 0; b < 2; ++b) Tile::zero_padding((role == 0 ? Qbuf : Dbuf) + b * TILE, tid_r);
  if (iters > 0) fetch(0, 0);
  settle_compiler_loads();                              // K / V fragments, lse, delta (and, with them, tile 0)
  bf16_t* my_p = Ps + (size_t)kb * (NQB * 2 * 64 * 8) + lane * 8;

  auto step = [&](int it, auto masked, auto parity) {
    constexpr bool MASKED = decltype(masked)::value;
    constexpr int PAR = decltype(parity)::value;
    const bf16_t* Qs = Qbuf + PAR * TILE;
    const bf16_t* Ds = Dbuf + PAR * TILE;
    const float* Ls = Lbuf + PAR * BK_Q;
    const float* Dl = Dlbuf + PAR * BK_Q;
    const bf16_t* rows_src = role == 0 ? Qs : Ds;       // phase 1 operand: Q (S) or dO (dP)
    const bf16_t* cols_src = role == 0 ? Ds : Qs;       // phase 2 operand: dO^T (dV) or Q^T (dK)
    if (tid < BK_Q) { Lbuf[PAR * BK_Q + tid] = st_l * LOG2E; Dlbuf[PAR * BK_Q + tid] = st_d; }
    // tile `it` is there for everyone, and everyone is done with tile it-1 and its P
    wait_async_tiles();
    __syncthreads();
    if (it + 1 < iters) fetch(it + 1, 1 - PAR);
    const int q0 = qstart + (it % nqt) * BK_Q;
    // phase 1: X[q, key] = rows(Q or dO) . (K or V)^T for both 32-query blocks
    f32x16 xacc[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) xacc[qb][r] = 0.f;
    {
      constexpr int NSTEP = NQB * KS, AHEAD = 2;
      bf16x8 fx[AHEAD + 1];
#pragma unroll
      for (int n = 0; n < AHEAD && n < NSTEP; ++n) fx[n] = frag_rows<DHL>(rows_src, (n / KS) * 32, n % KS, lane);
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) {
        const int m = n + AHEAD;
        if (m < NSTEP) fx[m % (AHEAD + 1)] = frag_rows<DHL>(rows_src, (m / KS) * 32, m % KS, lane);
        xacc[n / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[n % (AHEAD + 1)], kvf[n % KS], xacc[n / KS], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    bf16x8 op[NQB][2];                                  // B operands of phase 2: P (role 0) or dS (role 1)
    if (role == 0) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int qoff = qb * 32 + g * 8 + half * 4;
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(Ls + qoff);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = g * 4 + e;
            float p = __builtin_amdgcn_exp2f(fmaf(xacc[qb][r], scale_log2, -l4[e]));
            if (MASKED) {
              const int qi = q0 + qoff + e;
              if (qi >= Lq || kpos >= L || (CAUSAL && kpos > qi)) p = 0.f;
            }
            xacc[qb][r] = p;
          }
        }
        op[qb][0] = acc_to_operand(xacc[qb], 0);
        op[qb][1] = acc_to_operand(xacc[qb], 1);
        *reinterpret_cast<bf16x8*>(my_p + (qb * 2 + 0) * 64 * 8) = op[qb][0];
        *reinterpret_cast<bf16x8*>(my_p + (qb * 2 + 1) * 64 * 8) = op[qb][1];
      }
    }
    __syncthreads();                                    // P of this step is in LDS
    if (role == 1) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const bf16x8 pa = *reinterpret_cast<const bf16x8*>(my_p + (qb * 2 + 0) * 64 * 8);
        const bf16x8 pb = *reinterpret_cast<const bf16x8*>(my_p + (qb * 2 + 1) * 64 * 8);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(Dl + qb * 32 + g * 8 + half * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = g * 4 + e;
            const float p = (float)(r < 8 ? pa[r] : pb[r - 8]);
            xacc[qb][r] = p * (xacc[qb][r] - d4[e]);
          }
        }
        op[qb][0] = acc_to_operand(xacc[qb], 0);
        op[qb][1] = acc_to_operand(xacc[qb], 1);
      }
    }
    // phase 2: acc^T[c, key] += cols(dO or Q)^T . (P or dS), transposed operands requested one pair ahead
    {
      constexpr int NSTEP = NQB * NB;
      bf16x8 fr[2][2];
      fr[0][0] = frag_cols<DHL>(cols_src, 0, 0, lane);
      fr[0][1] = frag_cols<DHL>(cols_src, 0, 16, lane);
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) {
        const int qb = n / NB, j = n % NB, m = n + 1;
        if (m < NSTEP) {
          fr[m & 1][0] = frag_cols<DHL>(cols_src, (m % NB) * 32, (m / NB) * 32, lane);
          fr[m & 1][1] = frag_cols<DHL>(cols_src, (m % NB) * 32, (m / NB) * 32 + 16, lane);
        }
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n & 1][0], op[qb][0], acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n & 1][1], op[qb][1], acc[j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // which query tiles need the mask tests: as in the single-wavefront kernel, per 32-key block
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  auto step_of = [&](int it, bool masked) {
    if (it & 1) { if (masked) step(it, std::true_type{}, P1{}); else step(it, std::false_type{}, P1{}); }
    else { if (masked) step(it, std::true_type{}, P0{}); else step(it, std::false_type{}, P0{}); }
  };
  {
    // (one call site per copy of the step: with two the compiler stops inlining them)
    const bool all_masked = kb0 + BK_KEYS > L;
    const int n_front = CAUSAL ? min(nqt, (kb * 32 + 32 + BK_Q - 1) / BK_Q) : 0;
    const int n_whole = max(n_front, (Lq - qstart) % BK_Q ? nqt - 1 : nqt);
    for (int it = 0, t = 0; it < iters; ++it, t = (t + 1 == nqt ? 0 : t + 1))
      step_of(it, all_masked || t < n_front || t >= n_whole);
  }
  const float out_scale = role == 0 ? 1.0f : scale;     // dV as it is, dK times the softmax scale
  if (kpos < L && gsplit > 1) {
    const size_t plane = (size_t)Ttot * Hkv * DH;
    float* pp = part + ((size_t)gs * 2 + (role == 0 ? 1 : 0)) * plane + (size_t)(lo + kpos) * (Hkv * DH) + hk * DH;
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH)
          *reinterpret_cast<f32x4*>(pp + j * 32 + g * 8 + half * 4) =
              f32x4{acc[j][g * 4] * out_scale, acc[j][g * 4 + 1] * out_scale, acc[j][g * 4 + 2] * out_scale,
                    acc[j][g * 4 + 3] * out_scale};
  } else if (kpos < L) {
    bf16_t* pp = (role == 0 ? dv : dk) + (size_t)(lo + kpos) * ldd + hk * DH;
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(acc[j][g * 4 + e] * out_scale);
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH)
          *reinterpret_cast<bf16x4*>(pp + j * 32 + g * 8 + half * 4) = w;
      }
  }
}

// dQ of one 128-row query tile of one q head: walks the key tiles, scores kept as
// S^T[key, q] as in the forward kernel.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void fa_bwd_dq_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int ld,
    int ldk, const bf16_t* __restrict__ d_o, int ldo, const float* __restrict__ lse,
    const float* __restrict__ delta, const int32_t* __restrict__ cu, const int32_t* __restrict__ cuk,
    int S, bf16_t* __restrict__ dq, int ldd, int Ttot, int Hq, int group, float scale, float scale_log2,
    SeqOrder ord) {
  // K and V tiles are double-buffered and streamed into LDS as in the forward kernel; Q and dO of
  // this wavefront's 32 queries stay in registers.  At head size 128 a step is one 32-key block:
  // with two blocks' fragments and masks in flight next to Q, dO and the dQ accumulator the
  // kernel spills at two wavefronts per SIMD.  (dO read from LDS instead, a quarter more fragment
  // reads per key block, measured 1 % slower.)
  constexpr int FKD = DH > 72 ? 32 : FK;
  constexpr int TILE = FKD * HeadDim<DH>::DHL;
  __shared__ __attribute__((aligned(1024))) bf16_t Kbuf[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vbuf[2 * TILE];
  int seq, qt, nqt, tile_id, hq;
  tile_and_head(Hq, &tile_id, &hq);
  if (!find_tile(cu, ord, S, FQ, tile_id, &seq, &qt, &nqt)) return;
  const int hk = hq / group;
  const int lo = cu[seq], L = cu[seq + 1] - lo;
  const int lok = cuk[seq], Lk = cuk[seq + 1] - lok;
  const int q0 = qt * FQ;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int qpos = q0 + wave * 32 + (lane & 31);
  const int qrow = min(qpos, L - 1);
  if (Lk == 0) {
    // no key in this chunk (workgroup-uniform): dq = 0
    if (qpos < L) {
      bf16_t* pq = dq + (size_t)(lo + qpos) * ldd + hq * DH;
      for (int c = half * (DH / 2); c < (half + 1) * (DH / 2); c += 4) {
        bf16x4 z = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
        *reinterpret_cast<bf16x4*>(pq + c) = z;
      }
    }
    return;
  }

  bf16x8 qf[HeadDim<DH>::KS], dof[HeadDim<DH>::KS];
  {
    const bf16_t* qp = q + (size_t)(lo + qrow) * ld + hq * DH;
    const bf16_t* dp = d_o + (size_t)(lo + qrow) * ldo + hq * DH;
#pragma unroll
    for (int ks = 0; ks < HeadDim<DH>::KS; ++ks) {
      qf[ks] = load_chunk<DH>(qp, ks * 2 + half);
      dof[ks] = load_chunk<DH>(dp, ks * 2 + half);
    }
  }
  const float my_lse = lse[(size_t)hq * Ttot + lo + qrow] * LOG2E;
  const float my_delta = delta[(size_t)hq * Ttot + lo + qrow];
  f32x16 dqacc[HeadDim<DH>::NB];
#pragma unroll
  for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[j][r] = 0.f;

  const int kend = CAUSAL ? min(Lk, q0 + FQ) : Lk;
  const int nkt = (kend + FKD - 1) / FKD;
  const bf16_t* kbase = k + (size_t)lok * ldk + hk * DH;
  const bf16_t* vbase = v + (size_t)lok * ldk + hk * DH;
  using Tile = TileAsync<FKD, DH, 256>;
  Tile tile;
  tile.init(ldk, tid);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    Tile::zero_padding(Kbuf + b * TILE, tid);
    Tile::zero_padding(Vbuf + b * TILE, tid);
  }
  tile.issue(kbase, ldk, Lk, Kbuf, wave_u);
  tile.issue(vbase, ldk, Lk, Vbuf, wave_u);
  settle_compiler_loads();                 // the Q and dO fragments, lse, delta (and, with them, tile 0)
  // two copies of the step, without and with the mask test, as in the forward kernel
  constexpr bool FOLD_DELTA = DH <= 64;      // dP accumulators start at -delta (see the dK/dV kernel)
  auto step = [&](int kt, auto masked, auto parity) {
    constexpr bool MASKED = decltype(masked)::value;
    constexpr int PAR = decltype(parity)::value;
    const bf16_t* Ks = Kbuf + PAR * TILE;
    const bf16_t* Vs = Vbuf + PAR * TILE;
    wait_async_tiles();
    __syncthreads();      // tile kt is there for everyone, and everyone is done with tile kt-1
    if (kt + 1 < nkt) {
      const size_t next = (size_t)(kt + 1) * FKD * ldk;
      tile.issue(kbase + next, ldk, Lk - (kt + 1) * FKD, Kbuf + (1 - PAR) * TILE, wave_u);
      tile.issue(vbase + next, ldk, Lk - (kt + 1) * FKD, Vbuf + (1 - PAR) * TILE, wave_u);
    }
    const int key0 = kt * FKD;
    // S^T = K Q^T and dP^T = V dO^T of BP 32-key blocks are issued before any softmax arithmetic,
    // so that one block's MFMAs run under the other's vector work; at head size 128 that is one
    // block at a time (two sets of accumulators do not fit next to two resident wavefronts).
    constexpr int NBLK = FKD / 32, BP = DH > 72 ? 1 : NBLK, KS = HeadDim<DH>::KS;
#pragma unroll
    for (int b0 = 0; b0 < NBLK; b0 += BP) {
      f32x16 sacc[BP], dpacc[BP];
#pragma unroll
      for (int bi = 0; bi < BP; ++bi)
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[bi][r] = 0.f; dpacc[bi][r] = FOLD_DELTA ? -my_delta : 0.f; }   // MFMAs leave dP - delta
      {
        // operand fragments are requested AHEAD MFMA pairs before their use (see the dK/dV kernel)
        constexpr int NSTEP = BP * KS, AHEAD = 2;
        bf16x8 fk[AHEAD + 1], fv[AHEAD + 1];
        auto request = [&](int n) {
          fk[n % (AHEAD + 1)] = frag_rows<HeadDim<DH>::DHL>(Ks, (b0 + n / KS) * 32, n % KS, lane);
          fv[n % (AHEAD + 1)] = frag_rows<HeadDim<DH>::DHL>(Vs, (b0 + n / KS) * 32, n % KS, lane);
        };
#pragma unroll
        for (int n = 0; n < AHEAD && n < NSTEP; ++n) request(n);
#pragma unroll
        for (int n = 0; n < NSTEP; ++n) {
          const int bi = n / KS, ks = n % KS;
          if (n + AHEAD < NSTEP) request(n + AHEAD);
          sacc[bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[n % (AHEAD + 1)], qf[ks], sacc[bi], 0, 0, 0);
          dpacc[bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[n % (AHEAD + 1)], dof[ks],
                                                              dpacc[bi], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int bi = 0; bi < BP; ++bi) {
        const int b = b0 + bi;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[bi][r], scale_log2, -my_lse));
          if (MASKED) {
            const int key = key0 + b * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (key >= Lk || (CAUSAL && key > qpos)) p = 0.f;
          }
          dpacc[bi][r] = FOLD_DELTA ? p * dpacc[bi][r] : p * (dpacc[bi][r] - my_delta);
        }
        const bf16x8 s0 = acc_to_operand(dpacc[bi], 0), s1 = acc_to_operand(dpacc[bi], 1);
        {
          // dQ += dS K, the transposed K operands requested one pair of MFMAs ahead
          constexpr int NB = HeadDim<DH>::NB;
          bf16x8 fr[2][2];
          fr[0][0] = frag_cols<HeadDim<DH>::DHL>(Ks, 0, b * 32, lane);
          fr[0][1] = frag_cols<HeadDim<DH>::DHL>(Ks, 0, b * 32 + 16, lane);
#pragma unroll
          for (int j = 0; j < NB; ++j) {
            if (j + 1 < NB) {
              fr[(j + 1) & 1][0] = frag_cols<HeadDim<DH>::DHL>(Ks, (j + 1) * 32, b * 32, lane);
              fr[(j + 1) & 1][1] = frag_cols<HeadDim<DH>::DHL>(Ks, (j + 1) * 32, b * 32 + 16, lane);
            }
            dqacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][0], s0, dqacc[j], 0, 0, 0);
            dqacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 1][1], s1, dqacc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  };
  int n_plain = Lk / FKD;
  if (CAUSAL) n_plain = min(n_plain, (q0 + wave * 32 + 1) / FKD);
  n_plain = min(n_plain, nkt);
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  for (int kt = 0; kt < nkt; ++kt) {
    const bool plain = kt < n_plain;
    if (kt & 1) { if (plain) step(kt, std::false_type{}, P1{}); else step(kt, std::true_type{}, P1{}); }
    else { if (plain) step(kt, std::false_type{}, P0{}); else step(kt, std::true_type{}, P0{}); }
  }
  if (qpos < L) {
    bf16_t* pq = dq + (size_t)(lo + qpos) * ldd + hq * DH;
#pragma unroll
    for (int j = 0; j < HeadDim<DH>::NB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(dqacc[j][g * 4 + e] * scale);
        if (DH % 32 == 0 || j * 32 + g * 8 + half * 4 < DH)
          *reinterpret_cast<bf16x4*>(pq + j * 32 + g * 8 + half * 4) = w;
      }
  }
}

// dk, dv = sum over the q-head parts of the fp32 partials, in part order
__global__ void fa_dkdv_reduce_kernel(const float* __restrict__ part, int gsplit, int Ttot, int W /* Hkv*dh */,
                                      bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int ldd) {
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const long plane = (long)Ttot * W;
  if (i >= plane) return;
  const int t = (int)(i / W), c = (int)(i % W);
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < gsplit; ++g) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(part + ((size_t)g * 2 + which) * plane + i);
      s[0] += v[0]; s[1] += v[1]; s[2] += v[2]; s[3] += v[3];
    }
    bf16x4 w = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
    *reinterpret_cast<bf16x4*>((which == 0 ? dk : dv) + (size_t)t * ldd + c) = w;
  }
}

// q-head parts per kv head in the dK/dV kernel: more workgroups when few key tiles x kv
// heads would leave most CUs idle (grouped-query attention over a short pack)
int dkdv_group_split(int tiles, int Hkv, int group) {
  const long wgs = (long)tiles * Hkv;
  int want = (int)((1024 + wgs - 1) / wgs);
  int gsplit = 1;
  for (int s = 1; s <= group; ++s)
    if (group % s == 0 && s <= want) gsplit = s;
  return gsplit;
}

template <int DH>
bm_status bwd_launch(const AttnArgs& a, const void* o, const void* d_o, const float* lse, void* dq,
                     void* dk, void* dv, int ldd, float* delta, hipStream_t st) {
  const int ldo = a.Hq * a.dh;
  const int ldd_kv = a.ld_dkv ? a.ld_dkv : ldd;
  const float scale = 1.0f / sqrtf((float)a.dh);
  const float sl2 = scale * LOG2E;
  const long n = (long)a.T * a.Hq;
  if (n > 0)
    hipLaunchKernelGGL((fa_delta_kernel<DH>), dim3(cdiv(n * DeltaLanes<DH>::N, 256)), dim3(256), 0, st, (const bf16_t*)o,
                       (const bf16_t*)d_o, ldo, delta, a.T, a.Hq);
  const int ktiles = count_tiles(a.kv_cu_host(), a.S, BK_KEYS);
  const int gsplit = ktiles > 0 ? dkdv_group_split(ktiles, a.Hkv, a.Hq / a.Hkv) : 1;
  float* part = delta + align_up((size_t)a.Hq * a.T, 64);      // after the delta plane
  const int Tk = a.kv_T();
  dim3 gkv(ktiles * a.Hkv * gsplit), gq(count_tiles(a.cu_host, a.S, FQ) * a.Hq);
  // a key tile runs as long as its sequence has queries, a query tile as long as it has keys
  const SeqOrder ord_kv = make_seq_order(a.kv_cu_host(), a.cu_host, a.S, BK_KEYS, !a.causal);
  const SeqOrder ord_q = make_seq_order(a.cu_host, a.kv_cu_host(), a.S, FQ, !a.causal);
#define BM_L(C)                                                                                  \
  if (ktiles > 0 && DH > 64)                                                                     \
    hipLaunchKernelGGL((fa_bwd_dkdv_pair_kernel<(DH > 64 ? DH : 128), C>), gkv, dim3(512), 0, st, \
                       (const bf16_t*)a.q,                                                       \
                       (const bf16_t*)a.k, (const bf16_t*)a.v, a.ld_qkv, a.kv_ld(),              \
                       (const bf16_t*)d_o, ldo, lse, delta, a.cu_dev, a.kv_cu_dev(), a.S,        \
                       (bf16_t*)dk, (bf16_t*)dv, ldd_kv, a.T, Tk, a.Hkv, a.Hq / a.Hkv, scale, sl2, \
                       gsplit, part, ord_kv);                                                    \
  else if (ktiles > 0)                                                                           \
    hipLaunchKernelGGL((fa_bwd_dkdv_kernel<DH, C>), gkv, dim3(256), 0, st, (const bf16_t*)a.q,    \
                       (const bf16_t*)a.k, (const bf16_t*)a.v, a.ld_qkv, a.kv_ld(),              \
                       (const bf16_t*)d_o, ldo, lse, delta, a.cu_dev, a.kv_cu_dev(), a.S,        \
                       (bf16_t*)dk, (bf16_t*)dv, ldd_kv, a.T, Tk, a.Hkv, a.Hq / a.Hkv, scale, sl2, \
                       gsplit, part, ord_kv);                                                    \
  if (gq.x > 0)                                                                                  \
    hipLaunchKernelGGL((fa_bwd_dq_kernel<DH, C>), gq, dim3(256), 0, st, (const bf16_t*)a.q,      \
                       (const bf16_t*)a.k, (const bf16_t*)a.v, a.ld_qkv, a.kv_ld(),              \
                       (const bf16_t*)d_o, ldo, lse, delta, a.cu_dev, a.kv_cu_dev(), a.S,        \
                       (bf16_t*)dq, ldd, a.T, a.Hq, a.Hq / a.Hkv, scale, sl2, ord_q)
  if (a.causal) { BM_L(true); } else { BM_L(false); }
#undef BM_L
  if (gsplit > 1 && ktiles > 0) {
    const long n4 = (long)Tk * a.Hkv * a.dh / 4;
    hipLaunchKernelGGL(fa_dkdv_reduce_kernel, dim3(cdiv(n4, 256)), dim3(256), 0, st, part, gsplit, Tk,
                       a.Hkv * a.dh, (bf16_t*)dk, (bf16_t*)dv, ldd_kv);
  }
  BM_CHECK_LAUNCH("fa_bwd");
  return BM_OK;
}

}  // namespace

bool attention_mfma_supported(const AttnArgs& a) {
  return a.dtype == BM_DTYPE_BF16 && (a.dh == 64 || a.dh == 72 || a.dh == 128) && a.ld_qkv % 8 == 0 &&
         a.kv_ld() % 8 == 0;
}

bm_status attention_forward_mfma(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
  if (a.dh == 128) return fwd_launch<128>(a, o, lse, st);
  if (a.dh == 72) return fwd_launch<72>(a, o, lse, st);
  return fwd_launch<64>(a, o, lse, st);
}

size_t attention_backward_mfma_scratch_bytes(int Hq, int Hkv, int dh, int Tq, int Tk) {
  // the delta plane of the query rows, then room for the fp32 dK/dV partials of the largest
  // q-head split
  const size_t delta = align_up((size_t)Hq * Tq, 64) * sizeof(float);
  const int group = Hq / Hkv;
  const size_t part = group > 1 ? (size_t)group * 2 * Tk * Hkv * dh * sizeof(float) : 0;
  return align_up(delta + part, 256);
}

bm_status attention_backward_mfma(const AttnArgs& a, const void* o, const void* d_o, const float* lse,
                                  void* dq, void* dk, void* dv, int ld_dqkv, void* scratch,
                                  size_t, hipStream_t st) {
  if (a.dh == 128) return bwd_launch<128>(a, o, d_o, lse, dq, dk, dv, ld_dqkv, (float*)scratch, st);
  if (a.dh == 72) return bwd_launch<72>(a, o, d_o, lse, dq, dk, dv, ld_dqkv, (float*)scratch, st);
  return bwd_launch<64>(a, o, d_o, lse, dq, dk, dv, ld_dqkv, (float*)scratch, st);
}

}  // namespace bm
