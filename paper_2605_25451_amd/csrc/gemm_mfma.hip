// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   NT: C[M,N]  = A[M,K] B[N,K]^T (+bias)(+residual)   linear forward
//   NN: C[M,N]  = A[M,K] B[K,N]                        input gradient
//   TN: C[M,N] += A[K,M]^T B[K,N]     (C fp32)         weight gradient
//
// One workgroup owns a BM x BN tile of C and walks K in slices of BK=64.  Both
// operand slices are staged in LDS (two buffers: the next slice is fetched
// from HBM into registers while the current one feeds the MFMAs, one barrier per
// slice).  An operand whose K index is contiguous in memory is kept as
// [row][k] with its 16-byte chunks XOR-swizzled by the row, and fragments are
// read with ds_read_b128.  An operand whose K index is the slow one (B of NN,
// both operands of TN) is kept as [k][row] and fragments are read with the
// LDS transpose read (ds_read_b64_tr_b16), so no transposed copy is ever made.
// Workgroup ids are remapped so that the workgroups of one XCD (they share an
// L2) cover a compact block of tiles.  The K split of TN writes fp32 partial
// tiles that a second kernel sums in a fixed order: no floating-point atomics.
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

constexpr int BK = 64;          // k slice
constexpr int KCH = BK / 8;     // 16-byte chunks per k-contiguous row

struct GemmParams {
  const bf16_t* A; const bf16_t* B; void* C;
  const bf16_t* bias; const bf16_t* residual;
  const bf16_t* sw_up = nullptr; bf16_t* sw_dup = nullptr; bf16_t* sw_a = nullptr;   // SwiGLU backward epilogue (see GemmEpilogue)
  bf16_t* swf_a = nullptr;      // SwiGLU forward epilogue (see GemmEpilogue); N = 2F
  float* partial;               // TN with splits > 1
  int M, N, K, lda, ldb, ldc;
  int tiles_m, tiles_n, splits, k_per_split;
  int out_fp32;
  int xcd_split;                // each k split owns 8/splits XCDs (splits in {2,4,8})
  // grouped problems (see GemmGroups); all null / zero otherwise
  const int32_t* tile_group;
  const int32_t* group_rows;
  long b_group_stride, c_group_stride;
  int grid_groups;              // host: workgroups = tiles * splits * grid_groups (>= 1)
  // paired launch: workgroups pair_wgs0.. of the grid work on a second problem of the same
  // kind and the same K (two weight gradients that each leave CUs idle share one grid)
  int pair_wgs0;                // 0: one problem
  struct Second {
    const bf16_t* A; const bf16_t* B; void* C; float* partial;
    int M, N, lda, ldb, ldc, tiles_m, tiles_n, splits, k_per_split, xcd_split;
  } second;
};

// ---- LDS layouts ---------------------------------------------------------
// k-contiguous operand: [rows][KCH chunks]; chunk c of row r sits at c ^ ((r>>1)&7).
__device__ inline int kc_offset(int row, int c) {          // in bf16 elements
  return row * BK + ((c ^ ((row >> 1) & (KCH - 1))) << 3);
}
// transposed operand: [BK k-rows][R/8 chunks]; chunk c of k-row k sits at
// c ^ ((k&3)<<2) ^ (((k>>3)&1)<<1): a transpose read touches 4 consecutive k-rows x 32 bytes
// per 16 lanes; the first term puts the 4 k-rows into different 64-byte bank windows, the
// second moves the lane group that reads 8 k-rows further on into the other half of each.
template <int R>
__device__ inline int tr_offset(int k, int c) {             // in bf16 elements
  const int pos = c ^ ((k & 3) << 2) ^ (((k >> 3) & 1) << 1);
  return k * R + (pos << 3);
}

template <int R>
__device__ inline bf16x8 tr_fragment(const bf16_t* lds, int row0, int k0, int lane) {
  // 32(row) x 16(k) fragment of an operand stored [k][row]; lane l gets row
  // row0 + l%32 and k = k0 + (l/32)*8 .. +7
  const int gi = lane >> 4, s = lane & 15;
  const int r = row0 + (gi & 1) * 16 + (s & 3) * 4;        // 4 consecutive rows (8 bytes)
  const int k = k0 + (gi >> 1) * 8 + (s >> 2);
  const int c = r >> 3, within = r & 7;
  const bf16_t* p0 = lds + tr_offset<R>(k, c) + within;
  const bf16_t* p1 = lds + tr_offset<R>(k + 4, c) + within;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p1);
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

__device__ inline bf16x8 kc_fragment(const bf16_t* lds, int row0, int ks, int lane) {
  const int row = row0 + (lane & 31);
  const int c = ks * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(lds + kc_offset(row, c));
}

// 16(row) x 32(k) fragments of the v_mfma_f32_16x16x32_bf16 operands: lane l holds row
// row0 + l%16 and k = k0 + (l/16)*8 .. +7.
__device__ inline bf16x8 kc_fragment16(const bf16_t* lds, int row0, int ks32, int lane) {
  const int row = row0 + (lane & 15);
  const int c = ks32 * 4 + (lane >> 4);
  return *reinterpret_cast<const bf16x8*>(lds + kc_offset(row, c));
}

template <int R>
__device__ inline bf16x8 tr_fragment16(const bf16_t* lds, int row0, int k0, int lane) {
  // operand stored [k][row]: the 16 lanes of group gi read a 4(k) x 16(row) block, 8 bytes each, and
  // the transpose read hands lane s row row0 + s with 4 consecutive k; two reads give 8 k
  const int gi = lane >> 4, s = lane & 15;
  const int r = row0 + (s & 3) * 4;
  const int k = k0 + gi * 8 + (s >> 2);
  const int c = r >> 3, within = r & 7;
  const bf16_t* p0 = lds + tr_offset<R>(k, c) + within;
  const bf16_t* p1 = lds + tr_offset<R>(k + 4, c) + within;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p1);
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

// acc += a b^T with v_mfma_f32_16x16x32_bf16.  Written as an asm statement that ties the
// accumulator block to the accumulation half of the register file: with 64 four-register blocks
// the allocator otherwise keeps some of them in the other half and runs out of registers there
// (copies between the halves inside the loop, spills).  The accumulator of a block is next
// touched 63 MFMAs later, far beyond any wait state the instruction asks for.
__device__ inline void mfma16(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// acc = a b^T: the first product of a tile takes the constant 0 as its addend, so the accumulators
// are never initialised by separate instructions (which the compiler, not knowing that the asm
// statement is an MFMA, would place right in front of it without the wait states that needs)
__device__ inline void mfma16_first(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(acc) : "v"(a), "v"(b));
}

// ---- global -> registers -> LDS staging -----------------------------------
// Each thread moves CH = (R*BK/8)/NT chunks of 16 bytes per slice and operand.
// A chunk's position inside a slice never changes, so its global offset (relative
// to a wave-uniform slice base pointer that the caller advances) and its LDS offset
// are computed once; per slice a chunk costs one load and one LDS store.
template <int R, int NT, bool TR, bool KTAIL>
struct Stage {
  static constexpr int CH = (R * BK / 8) / NT;
  static constexpr int PARTS = BK / 32;          // one part per k-step (k = 32) of the MFMA loop
  static constexpr int PER = CH / PARTS;
  static_assert(CH % PARTS == 0, "tile does not split evenly over the k-steps");
  u32x4 v[CH];
  uint32_t goff[CH];    // byte offset from the slice base pointer
  unsigned live = 0u;   // KTAIL: bit i = chunk i lies inside the k range (else stored as zeros)
  // LDS byte offset of chunk i = soff[i & 1] + i * SSTRIDE: from one chunk of a thread to the next
  // the row (k-contiguous layout) or the k-row (transposed layout) advances by a fixed count that
  // leaves the XOR swizzle alone, except for bit 3 of the k-row, which alternates when that count is 8
  static constexpr int IROWS = TR ? NT / (R / 8) : NT / KCH;      // rows (k-rows) between chunks i and i+1
  static constexpr int SSTRIDE = IROWS * (TR ? R : BK) * 2;
  static constexpr bool ALT = TR && IROWS % 16 == 8;
  static_assert(TR ? IROWS % 8 == 0 : IROWS % 16 == 0, "the chunk stride would move the swizzle");
  uint32_t soff[ALT ? 2 : 1];

  // k index of chunk i inside a slice
  __device__ static inline int chunk_k(int i, int tid) {
    const int id = tid + i * NT;
    return TR ? id / (R / 8) : (id % KCH) * 8;
  }
  // rows_left: how many rows of the R dimension are valid from this tile's first row on
  // half > 0 (k-contiguous operand only): the tile's rows are gathered from two row ranges F rows
  // apart -- within every run of 2*half tile rows, the first half come from row0.. and the second
  // half from F + row0.. (the gate and the up half of a SwiGLU weight); offsets are then relative
  // to the matrix's first row
  __device__ inline void init(int ld, int rows_left, int tid, int half = 0, int F = 0, int row0 = 0) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int id = tid + i * NT;
      if (!TR && half > 0) {
        const int r = id / KCH;
        const int row = (r / half & 1) * F + row0 + (r / (2 * half)) * half + r % half;
        goff[i] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(id % KCH) * 8u) * 2u;
        continue;
      }
      if (TR) {            // memory [k][row]: chunk = 8 consecutive rows
        int row = (id % (R / 8)) * 8;
        if (row >= rows_left) row = 0;
        goff[i] = ((uint32_t)(id / (R / 8)) * (uint32_t)ld + (uint32_t)row) * 2u;
      } else {             // memory [row][k]: chunk = 8 consecutive k
        int row = id / KCH;
        if (row >= rows_left) row = rows_left - 1;
        goff[i] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(id % KCH) * 8u) * 2u;
      }
    }
#pragma unroll
    for (int i = 0; i < (ALT ? 2 : 1); ++i) {
      const int id = tid + i * NT;
      const int off = TR ? tr_offset<R>(id / (R / 8), id % (R / 8)) : kc_offset(id / KCH, id % KCH);
      soff[i] = (uint32_t)(off * 2 - i * SSTRIDE);
    }
  }

  // base: this tile's first row at the slice's first k (wave-uniform); k_left = valid k from there
  __device__ inline void load_one(int i, const bf16_t* __restrict__ base, int ld, int k_left, int tid) {
    uint32_t o = goff[i];
    if (KTAIL) {
      // keep the address valid and remember to store zeros instead
      const int kk = chunk_k(i, tid);
      const bool in = kk < k_left;
      live = (live & ~(1u << i)) | ((in ? 1u : 0u) << i);
      if (!in) o -= (TR ? (uint32_t)(kk - (k_left - 1)) * (uint32_t)ld : (uint32_t)(kk - (k_left - 8))) * 2u;
    }
    // the empty asm keeps the widening of the 32-bit offset next to the load, where the instruction
    // selector can fold it into the scalar-base + 32-bit-offset address form (hoisted out of the loop
    // it becomes a 64-bit register pair and a 64-bit add per load)
    asm volatile("" : "+v"(o));
    v[i] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(base) + o);
  }

  __device__ inline void store_one(int i, bf16_t* lds, int tid) const {
    (void)tid;
    u32x4 val = v[i];
    if (KTAIL && !((live >> i) & 1u)) val = u32x4{0u, 0u, 0u, 0u};
    *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(lds) + soff[ALT ? (i & 1) : 0] + i * SSTRIDE) = val;
  }

  __device__ inline void load(const bf16_t* __restrict__ base, int ld, int k_left, int tid) {
#pragma unroll
    for (int i = 0; i < CH; ++i) load_one(i, base, ld, k_left, tid);
  }
  __device__ inline void store(bf16_t* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < CH; ++i) store_one(i, lds, tid);
  }
};

// XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give
// each XCD a contiguous run of tiles, walked in column-major groups of GROUP_M
// tile rows (operand reuse in that XCD's L2).
__device__ inline void grouped_tile(int id, int tiles_m, int tiles_n, int* tm, int* tn) {
  constexpr int GROUP_M = 8;
  const int per_group = GROUP_M * tiles_n;
  const int g = id / per_group;
  const int first_m = g * GROUP_M;
  const int gsize = min(tiles_m - first_m, GROUP_M);
  const int in = id % per_group;
  *tm = first_m + in % gsize;
  *tn = in / gsize;
}

// K split with XCD affinity: split s owns the 8/splits XCDs s*G .. s*G+G-1 and each of
// them a contiguous run of that split's tiles, so an operand panel of one k range is
// fetched by as few L2s as possible (HBM traffic of the weight gradient is dominated by
// panels fetched once per XCD that touches them).
__device__ inline void split_tile_of_block(int pid, int tiles, int splits, int tiles_m, int tiles_n,
                                           int* split, int* tm, int* tn) {
  const int G = 8 / splits;
  const int xcd = pid & 7, local = pid >> 3;
  *split = xcd / G;
  grouped_tile((xcd % G) * (tiles / G) + local, tiles_m, tiles_n, tm, tn);
}

__device__ inline void tile_of_block(int pid, int total, int tiles_m, int tiles_n, int* tm, int* tn) {
  constexpr int XCDS = 8, GROUP_M = 4;     // measured: 4 tile rows per group is a little ahead of 8, 2 and 16
  int id = pid;
  if (total % XCDS == 0) id = (pid % XCDS) * (total / XCDS) + pid / XCDS;
  const int per_group = GROUP_M * tiles_n;
  const int g = id / per_group;
  const int first_m = g * GROUP_M;
  const int gsize = min(tiles_m - first_m, GROUP_M);
  const int in = id % per_group;
  *tm = first_m + in % gsize;
  *tn = in / gsize;
}

template <int BM, int BN, int WM, int WN, bool A_TR, bool B_TR, bool ACCUM_F32, bool KTAIL>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmParams p) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN_ = BN / WN;       // wave tile
  constexpr int FM = TM / 16, FN = TN_ / 16;       // 16x16 blocks per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int A_TILE = BM * BK, B_TILE = BN * BK;      // elements; buffers: A0 A1 B0 B1

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  int pid = blockIdx.x;
  if (p.pair_wgs0 > 0 && pid >= p.pair_wgs0) {
    // second problem of a paired launch (workgroup-uniform): take its description over
    pid -= p.pair_wgs0;
    p.A = p.second.A; p.B = p.second.B; p.C = p.second.C; p.partial = p.second.partial;
    p.M = p.second.M; p.N = p.second.N; p.lda = p.second.lda; p.ldb = p.second.ldb; p.ldc = p.second.ldc;
    p.tiles_m = p.second.tiles_m; p.tiles_n = p.second.tiles_n; p.splits = p.second.splits;
    p.k_per_split = p.second.k_per_split; p.xcd_split = p.second.xcd_split;
  }
  const int tiles = p.tiles_m * p.tiles_n;
  int split = pid / tiles;
  int tm, tn;
  if (p.xcd_split) split_tile_of_block(pid, tiles, p.splits, p.tiles_m, p.tiles_n, &split, &tm, &tn);
  else tile_of_block(pid % tiles, tiles, p.tiles_m, p.tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;
  int kbeg = split * p.k_per_split;
  int kend = min(p.K, kbeg + p.k_per_split);
  const bf16_t* Bmat = p.B;
  long c_off = 0;
  if (p.group_rows) {
    // grouped weight gradient: `split` is the group; its rows are the k range (all
    // wavefronts take the same exit: the values are workgroup-uniform)
    kbeg = min(p.group_rows[split], p.K);
    kend = min(p.group_rows[split + 1], p.K);
    if (kbeg >= kend) return;
    c_off = (long)split * p.c_group_stride;
    split = 0;
  } else if (p.tile_group) {
    const int g = p.tile_group[m0 / MOE_PAD];
    if (g < 0) return;
    Bmat += (long)g * p.b_group_stride;
  }

  f32x4 acc[FM][FN];        // first written by the first k-step of the first slice

  // Software pipeline, two slices deep: the registers of `sa`/`sb` always hold the
  // slice after the one being multiplied.  During k-step ks of slice j, part ks of
  // slice j+1 (fetched one whole slice ago) is written to the free LDS buffer and
  // the same registers are re-armed with part ks of slice j+2, so HBM/L2 latency is
  // covered by a full slice of MFMAs and memory instructions are spread between them.
  Stage<BM, NT, A_TR, KTAIL> sa;
  Stage<BN, NT, B_TR, KTAIL> sb;
  sa.init(p.lda, p.M - m0, tid);
  const bool swf = !B_TR && p.swf_a != nullptr;          // SwiGLU forward: N = 2F, a tile covers BN/2 columns of a
  if (swf) sb.init(p.ldb, BN, tid, TN_ / 2, p.N / 2, tn * (BN / 2));
  else sb.init(p.ldb, p.N - n0, tid);
  // slice base pointers (wave-uniform): first row of the tile at k = kbeg
  const bf16_t* a_base = A_TR ? p.A + (size_t)kbeg * p.lda + m0 : p.A + (size_t)m0 * p.lda + kbeg;
  const bf16_t* b_base = B_TR ? Bmat + (size_t)kbeg * p.ldb + n0 : Bmat + (swf ? (size_t)0 : (size_t)n0 * p.ldb) + kbeg;
  const size_t a_step = A_TR ? (size_t)BK * p.lda : (size_t)BK;
  const size_t b_step = B_TR ? (size_t)BK * p.ldb : (size_t)BK;
  sa.load(a_base, p.lda, kend - kbeg, tid);
  sb.load(b_base, p.ldb, kend - kbeg, tid);
  sa.store(smem, tid);
  sb.store(smem + 2 * A_TILE, tid);
  if (kbeg + BK < kend) {
    // same issue order as in the steady-state loop (part by part, A then B): the compiler's
    // wait-count bookkeeping merges this order with the loop's at the loop header, and any
    // difference makes the loop wait for younger loads than the one it stores
    constexpr int PA0 = Stage<BM, NT, A_TR, KTAIL>::PER, PB0 = Stage<BN, NT, B_TR, KTAIL>::PER;
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
#pragma unroll
      for (int i = 0; i < PA0; ++i) sa.load_one(ks * PA0 + i, a_base + a_step, p.lda, kend - kbeg - BK, tid);
#pragma unroll
      for (int i = 0; i < PB0; ++i) sb.load_one(ks * PB0 + i, b_base + b_step, p.ldb, kend - kbeg - BK, tid);
    }
  }
  __syncthreads();

  // one slice; NEXT1: the registers hold a slice to park, NEXT2: one more to fetch.
  // The flags are compile-time so that the steady-state loop body is branch-free
  // (the wait-count bookkeeping of the loads then stays exact across iterations).
  // Fragments.  A k-step (k = 32) is FM x FN MFMAs, row block i outermost: all FN B fragments
  // of a step are live (two register sets: the next step's are requested while this one runs),
  // the A fragments pass through a ring of four (the one for row block g+2 is requested when
  // row block g starts).  The last row block of a slice is held back: its operands are in
  // registers, so its MFMAs run AFTER the barrier that ends the slice and cover the LDS latency
  // of the next slice's first fragments.
  constexpr int KS32 = BK / 32, ROWS = KS32 * FM;
  static_assert(ROWS % 4 == 0, "the A ring continues across slices");
  bf16x8 ar[4], bfr[2][FN];
  auto pending_row = [&](auto&& between) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      mfma16(acc[FM - 1][j], bfr[(KS32 - 1) & 1][j], ar[(ROWS - 1) % 4]);
      between(j);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto slice = [&](auto next1_t, auto next2_t, auto pend_t, int k0, int cur) {
    constexpr bool NEXT1 = decltype(next1_t)::value, NEXT2 = decltype(next2_t)::value;
    constexpr bool PEND = decltype(pend_t)::value;
    const bf16_t* a_lds = smem + cur * A_TILE;
    const bf16_t* b_lds = smem + 2 * A_TILE + cur * B_TILE;
    bf16_t* a_nxt = smem + (cur ^ 1) * A_TILE;
    bf16_t* b_nxt = smem + 2 * A_TILE + (cur ^ 1) * B_TILE;
    auto a_frag = [&](int g) {
      const int ks = g / FM, r0 = wm * TM + (g % FM) * 16;
      return A_TR ? tr_fragment16<BM>(a_lds, r0, ks * 32, lane) : kc_fragment16(a_lds, r0, ks, lane);
    };
    auto b_frag = [&](int ks, int j) {
      const int r0 = wn * TN_ + j * 16;
      return B_TR ? tr_fragment16<BN>(b_lds, r0, ks * 32, lane) : kc_fragment16(b_lds, r0, ks, lane);
    };
    // the first MFMA of the slice waits for two fragments only: keep this request order
    ar[0] = a_frag(0);
    bfr[0][0] = b_frag(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    auto head_rest = [&](int n) {          // the other FN fragments of the head, one per call
      if (n + 1 < FN) bfr[0][n + 1] = b_frag(0, n + 1);
      else ar[1] = a_frag(1);
    };
    if (PEND) {
      pending_row(head_rest);
    } else {
#pragma unroll
      for (int n = 0; n < FN; ++n) head_rest(n);
      __builtin_amdgcn_sched_barrier(0);
    }
    // The other memory operations of a k-step -- the B fragment reads of the next step, the LDS
    // parks of this step's share of slice j+1 and the global loads that re-arm the same
    // registers with slice j+2 -- are dealt out evenly over the MFMAs and pinned there with
    // scheduling barriers so that they issue in the shadow of the matrix pipeline.
    constexpr int PA = Stage<BM, NT, A_TR, KTAIL>::PER, PB = Stage<BN, NT, B_TR, KTAIL>::PER;
    const bf16_t* a_g2 = a_base + (size_t)((k0 - kbeg) / BK + 2) * a_step;   // slice j+2
    const bf16_t* b_g2 = b_base + (size_t)((k0 - kbeg) / BK + 2) * b_step;
    const int k_left2 = kend - k0 - 2 * BK;
#pragma unroll
    for (int ks = 0; ks < KS32; ++ks) {
      const int nb = (ks + 1) & 1;
      const bool last = ks + 1 == KS32;
      // the last k-step has no fragments of a next step to fetch and one row block fewer to deal over
      const int SLOTS = last ? (FM - 1) * FN : FM * FN;
      const int FIRST = last ? FN : 0;                      // first op index of this step
      const int NOPS = FN + 2 * (PA + PB) - FIRST;
#pragma unroll
      for (int t = 0; t < SLOTS; ++t) {
        const int i = t / FN, j = t % FN, g = ks * FM + i;
        // operands swapped: the accumulator holds C^T blocks (see the epilogue)
        if (!PEND && ks == 0) mfma16_first(acc[i][j], bfr[ks & 1][j], ar[g % 4]);   // first slice of the tile
        else mfma16(acc[i][j], bfr[ks & 1][j], ar[g % 4]);
        if (j == 0 && g + 2 < ROWS) ar[(g + 2) % 4] = a_frag(g + 2);
#pragma unroll
        for (int oo = t * NOPS / SLOTS; oo < (t + 1) * NOPS / SLOTS; ++oo) {
          const int o = oo + FIRST;
          if (o < FN) {
            bfr[nb][o] = b_frag(ks + 1, o);
          } else if (o < FN + PA) {
            if (NEXT1) sa.store_one(ks * PA + (o - FN), a_nxt, tid);
          } else if (o < FN + PA + PB) {
            if (NEXT1) sb.store_one(ks * PB + (o - FN - PA), b_nxt, tid);
          } else if (o < FN + 2 * PA + PB) {
            if (NEXT2) sa.load_one(ks * PA + (o - FN - PA - PB), a_g2, p.lda, k_left2, tid);
          } else {
            if (NEXT2) sb.load_one(ks * PB + (o - FN - 2 * PA - PB), b_g2, p.ldb, k_left2, tid);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  };
  using yes = std::integral_constant<bool, true>;
  using no = std::integral_constant<bool, false>;
  {
    // the first slice has no row block pending; the flags of the steady-state slices are
    // compile-time constants, so the loop body is branch-free
    int cur = 0, k0 = kbeg;
    if (k0 + 2 * BK < kend) {
      slice(yes{}, yes{}, no{}, k0, cur); k0 += BK; cur ^= 1;
      for (; k0 + 2 * BK < kend; k0 += BK, cur ^= 1) slice(yes{}, yes{}, yes{}, k0, cur);
      slice(yes{}, no{}, yes{}, k0, cur); k0 += BK; cur ^= 1;
      slice(no{}, no{}, yes{}, k0, cur);
    } else if (k0 + BK < kend) {
      slice(yes{}, no{}, no{}, k0, cur); k0 += BK; cur ^= 1;
      slice(no{}, no{}, yes{}, k0, cur);
    } else {
      slice(no{}, no{}, no{}, k0, cur);
    }
    pending_row([](int) {});
    // the compiler does not know that the asm statements above are MFMAs and leaves no wait states
    // between the last of them and the epilogue's reads of the accumulators
    asm volatile("s_nop 15\n\ts_nop 15");
    __builtin_amdgcn_sched_barrier(0);
  }

  {
    // ---- epilogue.  The MFMAs ran with swapped operands, so block (i,j) holds C^T:
    // lane = row m = l%16, registers = 4 consecutive columns n = 4*(l/16) + e.
    // Each wavefront transposes its own 16-row strips through LDS (free after the last
    // barrier) and then writes whole rows: 16 bytes per lane, 256 contiguous bytes per row.
    constexpr int SLD = TN_ + 4;                         // padded fp32 row: conflict-free both ways
    float* stage = reinterpret_cast<float*>(smem_raw) + wave * (16 * SLD);
    constexpr int LPR = TN_ / 8;                          // lanes per output row (8 columns each)
    constexpr int RPI = 64 / LPR;                         // rows per store instruction
    static_assert(16 % RPI == 0, "a 16-row strip must be a whole number of store instructions");
    const int m_in = lane & 15, q4 = (lane >> 4) * 4;
    const int rcol = (lane % LPR) * 8, rrow = lane / LPR;
    const int gn = n0 + wn * TN_ + rcol;
    float bias[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bias[e] = 0.f;
    if (p.bias && gn < p.N) load16(p.bias + gn, bias);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      // SwiGLU backward epilogue: the saved g and u of this strip are requested before the
      // strip is transposed, so their latency is paid once per strip and not once per store
      Vec16<bf16_t> sw_g[16 / RPI], sw_u[16 / RPI];
      if (p.sw_up) {
#pragma unroll
        for (int t = 0; t < 16 / RPI; ++t) {
          const int gm = min(m0 + wm * TM + i * 16 + t * RPI + rrow, p.M - 1);
          const bf16_t* up = p.sw_up + (size_t)gm * (2 * p.N) + min(gn, p.N - 8);
          sw_g[t] = *reinterpret_cast<const Vec16<bf16_t>*>(up);
          sw_u[t] = *reinterpret_cast<const Vec16<bf16_t>*>(up + p.N);
        }
      }
#pragma unroll
      for (int j = 0; j < FN; ++j)
        *reinterpret_cast<f32x4*>(stage + m_in * SLD + j * 16 + q4) = acc[i][j];
      if (!A_TR && !B_TR && !ACCUM_F32 && p.swf_a) {
        // SwiGLU forward: the strip holds g in its first TN_/2 columns and u in the others, of the
        // same TN_/2 columns of a; a lane takes 8 of them
        constexpr int HW = TN_ / 2, LPR2 = HW / 8, RPI2 = 64 / LPR2;
        const int F = p.N / 2;
        const int rcol2 = (lane % LPR2) * 8, rrow2 = lane / LPR2;
        const int acol = tn * (BN / 2) + wn * HW + rcol2;
#pragma unroll
        for (int t = 0; t < (16 + RPI2 - 1) / RPI2; ++t) {
          const int row = t * RPI2 + rrow2;
          const int gm = m0 + wm * TM + i * 16 + row;
          if (row < 16 && gm < p.M) {
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(stage + row * SLD + rcol2);
            const f32x4 g1 = *reinterpret_cast<const f32x4*>(stage + row * SLD + rcol2 + 4);
            const f32x4 u0 = *reinterpret_cast<const f32x4*>(stage + row * SLD + HW + rcol2);
            const f32x4 u1 = *reinterpret_cast<const f32x4*>(stage + row * SLD + HW + rcol2 + 4);
            union { u32x4 v; bf16_t h[8]; } pg, pu, pa;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              pg.h[e] = Elt<bf16_t>::from_f(e < 4 ? g0[e] : g1[e - 4]);
              pu.h[e] = Elt<bf16_t>::from_f(e < 4 ? u0[e] : u1[e - 4]);
              const float g = (float)pg.h[e], u = (float)pu.h[e];
              const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
              pa.h[e] = Elt<bf16_t>::from_f(g * sig * u);
            }
            bf16_t* c = (bf16_t*)p.C + (size_t)gm * p.ldc + acol;
            __builtin_nontemporal_store(pg.v, reinterpret_cast<u32x4*>(c));
            __builtin_nontemporal_store(pu.v, reinterpret_cast<u32x4*>(c + F));
            *reinterpret_cast<u32x4*>(p.swf_a + (size_t)gm * F + acol) = pa.v;
          }
        }
        continue;
      }
#pragma unroll
      for (int t = 0; t < 16 / RPI; ++t) {
        const int row = t * RPI + rrow;
        const int gm = m0 + wm * TM + i * 16 + row;
        const f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * SLD + rcol);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * SLD + rcol + 4);
        if (gm < p.M && gn < p.N) {
          float out[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          const size_t idx = (size_t)gm * p.ldc + gn;
          if (ACCUM_F32) {
            // weight gradient: fp32, added to C (or parked as this split's partial tile)
            float* c = p.splits > 1 ? p.partial + ((size_t)split * p.M + gm) * p.N + gn
                                    : (float*)p.C + c_off + idx;
            f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
            if (p.splits == 1) {
              c0 = *reinterpret_cast<const f32x4*>(c);
              c1 = *reinterpret_cast<const f32x4*>(c + 4);
            }
            *reinterpret_cast<f32x4*>(c) = f32x4{c0[0] + out[0], c0[1] + out[1], c0[2] + out[2], c0[3] + out[3]};
            *reinterpret_cast<f32x4*>(c + 4) = f32x4{c1[0] + out[4], c1[1] + out[5], c1[2] + out[6], c1[3] + out[7]};
            continue;
          }
          if (p.sw_up) {
            // out = dA of 8 columns of one row: d_up and the activation instead of C
            const size_t up_idx = (size_t)gm * (2 * p.N) + gn;
            float dg[8], du[8], av[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float g = (float)sw_g[t].v[e], u = (float)sw_u[t].v[e];
              const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
              const float sl = g * sig;                          // silu(g)
              av[e] = sl * u;
              du[e] = out[e] * sl;
              dg[e] = out[e] * u * sig * (1.0f + g * (1.0f - sig));
            }
            store16(p.sw_dup + up_idx, dg);
            store16(p.sw_dup + up_idx + p.N, du);
            store16(p.sw_a + (size_t)gm * p.N + gn, av);
            continue;
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) out[e] += bias[e];
          if (p.residual) {
            float res[8];
            load16(p.residual + idx, res);
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] += res[e];
          }
          if (p.out_fp32) {
            float* c = (float*)p.C + idx;
            *reinterpret_cast<f32x4*>(c) = f32x4{out[0], out[1], out[2], out[3]};
            *reinterpret_cast<f32x4*>(c + 4) = f32x4{out[4], out[5], out[6], out[7]};
          } else {
            {
              union { u32x4 u; bf16_t h[8]; } pk;
#pragma unroll
              for (int e = 0; e < 8; ++e) pk.h[e] = Elt<bf16_t>::from_f(out[e]);
              __builtin_nontemporal_store(pk.u, reinterpret_cast<u32x4*>((bf16_t*)p.C + idx));
            }
          }
        }
      }
    }
  }
}

__global__ void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M, int N,
                                     float* __restrict__ C, int ldc) {
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= (long)M * N) return;
  const int m = (int)(i / N), n = (int)(i % N);
  float4 s = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < splits; ++k) {
    float4 v = *reinterpret_cast<const float4*>(partial + (size_t)k * M * N + i);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  float* c = C + (size_t)m * ldc + n;
  c[0] += s.x; c[1] += s.y; c[2] += s.z; c[3] += s.w;
}

struct Plan { int bm, bn, tiles_m, tiles_n, splits, k_per_split; };

constexpr int NUM_CU = 256;

// Tile size and K split from a small cost model in microseconds, calibrated on the
// weight-gradient shapes of the ViT-L and decoder blocks: workgroups run in rounds over
// the free slots (one 256x256 workgroup per CU, two 128x128 ones), each pays a fixed
// prologue/epilogue plus a per-slice time (1.85 us for a 256x256x64 slice, 1.25 us for a
// 128x128x64 slice that shares its CU with another workgroup), and a K split of the
// weight gradient pays for writing and re-reading its fp32 partial tiles.  Splits of 2, 4
// or 8 can be pinned to XCDs (see split_tile_of_block), which measures 4-7 % faster.
bool xcd_split_possible(int tiles, int splits) {
  return (splits == 2 || splits == 4 || splits == 8) && tiles % (8 / splits) == 0;
}

Plan make_plan(int layout, int M, int N, int K) {
  Plan best{};
  double best_t = 1e30;
  const int slices = cdiv(K, BK);
  for (int big = 1; big >= 0; --big) {
    const int tile = big ? 256 : 128;
    const double t_slice = big ? 1.85 : 1.25, t_fixed = big ? 8.0 : 4.0;
    const int slots = big ? NUM_CU : 2 * NUM_CU;
    const long tiles = (long)cdiv(M, tile) * cdiv(N, tile);
    const int max_split = layout == GEMM_TN ? (slices / 4 > 32 ? 32 : (slices / 4 < 1 ? 1 : slices / 4)) : 1;
    for (int sp = 1; sp <= max_split; ++sp) {
      const int per = cdiv(slices, sp);
      const int splits = cdiv(slices, per);
      if (splits != sp) continue;
      const long rounds = (tiles * splits + slots - 1) / slots;
      double t = rounds * (per * t_slice + t_fixed);
      if (splits > 1) t += 3.0 + 1.3 * splits * (double)M * N * 4.0 / 3.0e6;
      if (xcd_split_possible((int)tiles, splits)) t *= 0.95;
      if (t < best_t * 0.97) {            // prefer the earlier candidate on near ties
        best_t = t;
        best.bm = best.bn = tile;
        best.tiles_m = cdiv(M, tile); best.tiles_n = cdiv(N, tile);
        best.splits = splits; best.k_per_split = per * BK;
      }
    }
  }
  return best;
}

template <int BM, int BN, int WM, int WN, bool A_TR, bool B_TR, bool ACC, bool KTAIL>
bm_status launch_k(const GemmParams& p, hipStream_t st) {
  constexpr size_t lds_pipe = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
  constexpr size_t lds_epi = (size_t)WM * WN * 16 * (BN / WN + 4) * sizeof(float);
  constexpr size_t lds = lds_pipe > lds_epi ? lds_pipe : lds_epi;
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, A_TR, B_TR, ACC, KTAIL>;
  static bool attr_done = false;
  if (!attr_done) {
    BM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_done = true;
  }
  int wgs = p.tiles_m * p.tiles_n * p.splits * p.grid_groups;
  if (p.pair_wgs0 > 0) wgs = p.pair_wgs0 + p.second.tiles_m * p.second.tiles_n * p.second.splits;
  dim3 grid(wgs), block(WM * WN * 64);
  hipLaunchKernelGGL(kern, grid, block, lds, st, p);
  BM_CHECK_LAUNCH("gemm_mfma");
  return BM_OK;
}

// the zero-filling variant only when a k range is not a whole number of slices
template <int BM, int BN, int WM, int WN, bool A_TR, bool B_TR, bool ACC>
bm_status launch(const GemmParams& p, hipStream_t st) {
  if (p.K % BK) return launch_k<BM, BN, WM, WN, A_TR, B_TR, ACC, true>(p, st);
  return launch_k<BM, BN, WM, WN, A_TR, B_TR, ACC, false>(p, st);
}

}  // namespace

bool gemm_mfma_supported(int layout, int dtype, int M, int N, int K, int lda, int ldb, int ldc,
                         const GemmEpilogue& epi) {
  (void)epi;
  if (dtype != BM_DTYPE_BF16) return false;
  if (lda % 8 || ldb % 8) return false;                  // 16-byte rows
  if (N < 64) return false;                              // tiny problems: generic kernel
  if (layout == GEMM_TN) {
    // operands are [k][row]: rows come in chunks of 8, any k range of at least one chunk
    // works (a short one is zero-filled); one of M and K may be small (the 8..32-row
    // products of the adaLN modulation), not both
    if (M % 8 || N % 8 || ldc % 4) return false;
    return M >= 8 && K >= 8 && (M >= 64 || K >= 64);
  }
  // row-major A: rows past M are clamped to the last one and never stored, so few rows are fine
  if (M < 1 || K < 64) return false;
  return K % 8 == 0 && N % 8 == 0 && ldc % 8 == 0;          // 16-byte row chunks of C
}

size_t gemm_mfma_scratch_bytes(int layout, int M, int N, int K) {
  if (layout != GEMM_TN) return 0;
  Plan pl = make_plan(layout, M, N, K);
  return pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
}

bm_status gemm_mfma(int layout, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                    void* C, int ldc, const GemmEpilogue& epi, void* scratch, size_t scratch_bytes,
                    hipStream_t st) {
  Plan pl = make_plan(layout, M, N, K);
  GemmParams p;
  p.A = (const bf16_t*)A; p.B = (const bf16_t*)B; p.C = C;
  p.bias = (const bf16_t*)epi.bias; p.residual = (const bf16_t*)epi.residual;
  p.partial = (float*)scratch;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.tiles_m = pl.tiles_m; p.tiles_n = pl.tiles_n; p.splits = pl.splits; p.k_per_split = pl.k_per_split;
  p.out_fp32 = epi.out_fp32;
  p.sw_up = (const bf16_t*)epi.swiglu_up; p.sw_dup = (bf16_t*)epi.swiglu_dup; p.sw_a = (bf16_t*)epi.swiglu_a;
  p.swf_a = (bf16_t*)epi.swiglu_fwd_a;
  if (p.swf_a && (layout != GEMM_NT || N % 256 || epi.bias || epi.residual || epi.out_fp32)) {
    set_error("gemm: the SwiGLU forward epilogue needs the NT layout, N a multiple of 256 and no bias");
    return BM_ERR_INVALID_ARG;
  }
  p.tile_group = nullptr; p.group_rows = nullptr; p.b_group_stride = 0; p.c_group_stride = 0;
  p.grid_groups = 1; p.pair_wgs0 = 0; p.second = {};
  {
    p.xcd_split = xcd_split_possible(pl.tiles_m * pl.tiles_n, pl.splits) ? 1 : 0;
  }
  if (pl.splits > 1 && (!scratch || scratch_bytes < (size_t)pl.splits * M * N * sizeof(float))) {
    set_error("gemm TN: split reduction needs %zu scratch bytes, got %zu",
              (size_t)pl.splits * M * N * sizeof(float), scratch_bytes);
    return BM_ERR_WORKSPACE_TOO_SMALL;
  }
  bm_status rc;
  const bool big = pl.bm == 256;
  if (layout == GEMM_NT)
    rc = big ? launch<256, 256, 2, 2, false, false, false>(p, st) : launch<128, 128, 2, 2, false, false, false>(p, st);
  else if (layout == GEMM_NN)
    rc = big ? launch<256, 256, 2, 2, false, true, false>(p, st) : launch<128, 128, 2, 2, false, true, false>(p, st);
  else
    rc = big ? launch<256, 256, 2, 2, true, true, true>(p, st) : launch<128, 128, 2, 2, true, true, true>(p, st);
  BM_RETURN_IF(rc);
  if (layout == GEMM_TN && pl.splits > 1) {
    long n4 = ((long)M * N) / 4;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(cdiv(n4, 256)), dim3(256), 0, st,
                       (const float*)scratch, pl.splits, M, N, (float*)C, ldc);
    BM_CHECK_LAUNCH("splitk_reduce");
  }
  return BM_OK;
}

// common k split of a paired launch (0: the pair does not qualify)
static int pair_splits(int K, int M0, int N0, int M1, int N1) {
  if (K % BK || M0 < 256 || N0 < 256 || M1 < 256 || N1 < 256) return 0;
  const long tiles = (long)cdiv(M0, 256) * cdiv(N0, 256) + (long)cdiv(M1, 256) * cdiv(N1, 256);
  const int slices = K / BK;
  int sp = (int)(NUM_CU / tiles);
  if (sp > 32) sp = 32;
  if (sp > slices / 4) sp = slices / 4;
  for (; sp >= 1; --sp)
    if (cdiv(slices, cdiv(slices, sp)) == sp) break;
  return sp < 1 ? 0 : sp;
}

size_t gemm_mfma_tn_pair_scratch_bytes(int K, int M0, int N0, int M1, int N1) {
  const int sp = pair_splits(K, M0, N0, M1, N1);
  if (sp <= 1) return 0;
  return align_up((size_t)sp * M0 * N0 * sizeof(float), 256) + (size_t)sp * M1 * N1 * sizeof(float);
}

// Two weight gradients C_i[M_i,N_i] += A_i[K,M_i]^T B_i[K,N_i] over the same K in ONE grid, when
// both plans use 256x256 tiles and whole slices: a gradient whose tiles x splits do not fill
// the chip (1024x1024 next to 3072x1024 in a ViT-L block) no longer has the machine to itself.
// Returns false (nothing launched) when the pair does not qualify; the caller then runs two GEMMs.
bool gemm_mfma_tn_pair(int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0, void* C0, int ldc0,
                       int M1, int N1, const void* A1, int lda1, const void* B1, int ldb1, void* C1, int ldc1,
                       void* scratch, size_t scratch_bytes, hipStream_t st, bm_status* rc) {
  // rc == nullptr: only answer whether the pair qualifies
  const GemmEpilogue none;
  if (rc) *rc = BM_OK;
  if (K % BK) return false;
  if (!gemm_mfma_supported(GEMM_TN, BM_DTYPE_BF16, M0, N0, K, lda0, ldb0, ldc0, none) ||
      !gemm_mfma_supported(GEMM_TN, BM_DTYPE_BF16, M1, N1, K, lda1, ldb1, ldc1, none)) return false;
  // one plan for both: 256x256 tiles and the largest common k split whose workgroups fit the chip
  // in one round, so that all of them run equally long; it must beat the two separate plans
  const int sp = pair_splits(K, M0, N0, M1, N1);
  if (sp < 1) return false;
  const int slices = K / BK;
  Plan a{}, b{};
  a.bm = a.bn = b.bm = b.bn = 256;
  a.tiles_m = cdiv(M0, 256); a.tiles_n = cdiv(N0, 256);
  b.tiles_m = cdiv(M1, 256); b.tiles_n = cdiv(N1, 256);
  a.splits = b.splits = sp;
  a.k_per_split = b.k_per_split = cdiv(slices, sp) * BK;
  {
    const auto model = [&](int M, int N) {                      // what make_plan expects for one problem
      const Plan q = make_plan(GEMM_TN, M, N, K);
      const bool big = q.bm == 256;
      const long wg = (long)q.tiles_m * q.tiles_n * q.splits, slots = big ? NUM_CU : 2 * NUM_CU;
      double t = (double)((wg + slots - 1) / slots) * (q.k_per_split / BK * (big ? 1.85 : 1.25) + (big ? 8.0 : 4.0));
      if (q.splits > 1) t += 3.0 + 1.3 * q.splits * (double)M * N * 4.0 / 3.0e6;
      return t;
    };
    double together = a.k_per_split / BK * 1.85 + 8.0;
    if (sp > 1) together += 6.0 + 1.3 * sp * ((double)M0 * N0 + (double)M1 * N1) * 4.0 / 3.0e6;
    if (together >= model(M0, N0) + model(M1, N1)) return false;
  }
  const size_t part0 = a.splits > 1 ? align_up((size_t)a.splits * M0 * N0 * sizeof(float), 256) : 0;
  const size_t part1 = b.splits > 1 ? (size_t)b.splits * M1 * N1 * sizeof(float) : 0;
  if (part0 + part1 > scratch_bytes || (part0 + part1 > 0 && !scratch)) return false;
  const int wgs0 = a.tiles_m * a.tiles_n * a.splits;
  const bool xa = xcd_split_possible(a.tiles_m * a.tiles_n, a.splits), xb = xcd_split_possible(b.tiles_m * b.tiles_n, b.splits);
  if (xb && wgs0 % 8) return false;               // the second problem's XCD pinning needs an aligned start
  if (!rc) return true;
  GemmParams p;
  p.A = (const bf16_t*)A0; p.B = (const bf16_t*)B0; p.C = C0; p.bias = nullptr; p.residual = nullptr;
  p.partial = (float*)scratch;
  p.M = M0; p.N = N0; p.K = K; p.lda = lda0; p.ldb = ldb0; p.ldc = ldc0;
  p.tiles_m = a.tiles_m; p.tiles_n = a.tiles_n; p.splits = a.splits; p.k_per_split = a.k_per_split;
  p.out_fp32 = 0; p.xcd_split = xa ? 1 : 0;
  p.tile_group = nullptr; p.group_rows = nullptr; p.b_group_stride = 0; p.c_group_stride = 0; p.grid_groups = 1;
  p.pair_wgs0 = wgs0;
  p.second.A = (const bf16_t*)A1; p.second.B = (const bf16_t*)B1; p.second.C = C1;
  p.second.partial = (float*)((char*)scratch + part0);
  p.second.M = M1; p.second.N = N1; p.second.lda = lda1; p.second.ldb = ldb1; p.second.ldc = ldc1;
  p.second.tiles_m = b.tiles_m; p.second.tiles_n = b.tiles_n; p.second.splits = b.splits;
  p.second.k_per_split = b.k_per_split; p.second.xcd_split = xb ? 1 : 0;
  *rc = launch_k<256, 256, 2, 2, true, true, true, false>(p, st);
  if (*rc != BM_OK) return true;
  if (a.splits > 1)
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(cdiv((long)M0 * N0 / 4, 256)), dim3(256), 0, st, p.partial, a.splits,
                       M0, N0, (float*)C0, ldc0);
  if (b.splits > 1)
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(cdiv((long)M1 * N1 / 4, 256)), dim3(256), 0, st, p.second.partial,
                       b.splits, M1, N1, (float*)C1, ldc1);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) *rc = hip_fail(e, "splitk_reduce");
  return true;
}

bool gemm_mfma_grouped_supported(int layout, int dtype, int M, int N, int K, int lda, int ldb, int ldc) {
  if (dtype != BM_DTYPE_BF16) return false;
  if (N < 64 || lda % 8 || ldb % 8) return false;
  if (layout == GEMM_TN) return M >= 64 && M % 8 == 0 && N % 8 == 0 && ldc % 4 == 0 && K % MOE_PAD == 0;
  return K >= 64 && K % 8 == 0 && N % 8 == 0 && ldc % 8 == 0 && M % MOE_PAD == 0;
}

// 128x128 tiles: a row tile is one MOE_PAD block, so it never straddles two groups.
bm_status gemm_mfma_grouped(int layout, int M, int N, int K, const void* A, int lda, const void* B,
                            int ldb, void* C, int ldc, const GemmGroups& g, hipStream_t st,
                            const GemmEpilogue* epi) {
  static_assert(MOE_PAD == 128, "the grouped path uses 128-row tiles");
  GemmParams p;
  p.A = (const bf16_t*)A; p.B = (const bf16_t*)B; p.C = C;
  p.bias = nullptr; p.residual = nullptr; p.partial = nullptr;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.tiles_m = cdiv(M, 128); p.tiles_n = cdiv(N, 128); p.splits = 1; p.k_per_split = cdiv(K, BK) * BK;
  p.out_fp32 = 0; p.xcd_split = 0; p.pair_wgs0 = 0; p.second = {};
  p.tile_group = layout == GEMM_TN ? nullptr : g.tile_group;
  p.group_rows = layout == GEMM_TN ? g.group_rows : nullptr;
  p.b_group_stride = g.b_stride; p.c_group_stride = g.c_stride;
  p.grid_groups = layout == GEMM_TN ? g.n_groups : 1;
  if (epi) {
    // the SwiGLU epilogues ride on the 128x256 tiles (a tile gathers its weight rows per expert
    // exactly as the dense kernel does per matrix)
    const bool fwd = epi->swiglu_fwd_a != nullptr, bwd = epi->swiglu_up != nullptr;
    if (epi->bias || epi->residual || epi->out_fp32 || fwd == bwd || N % 256 || (fwd && layout != GEMM_NT) ||
        (bwd && (layout != GEMM_NN || !epi->swiglu_dup || !epi->swiglu_a))) {
      set_error("grouped gemm: only the SwiGLU epilogues (forward on NT, backward on NN, N a multiple of 256)");
      return BM_ERR_INVALID_ARG;
    }
    p.sw_up = (const bf16_t*)epi->swiglu_up; p.sw_dup = (bf16_t*)epi->swiglu_dup; p.sw_a = (bf16_t*)epi->swiglu_a;
    p.swf_a = (bf16_t*)epi->swiglu_fwd_a;
  }
  if ((layout == GEMM_TN ? p.group_rows == nullptr || g.n_groups < 1 : p.tile_group == nullptr)) {
    set_error("grouped gemm: group tables are NULL");
    return BM_ERR_INVALID_ARG;
  }
  // row tiles are pinned to 128 rows (one MOE_PAD block); 256 columns per tile where the output is
  // wide enough: per flop a 128x256 tile writes and reads a quarter less LDS than two 128x128 ones
  if (layout != GEMM_TN && N >= 256) {
    p.tiles_n = cdiv(N, 256);
    if (layout == GEMM_NT) return launch<128, 256, 2, 2, false, false, false>(p, st);
    return launch<128, 256, 2, 2, false, true, false>(p, st);
  }
  if (layout == GEMM_NT) return launch<128, 128, 2, 2, false, false, false>(p, st);
  if (layout == GEMM_NN) return launch<128, 128, 2, 2, false, true, false>(p, st);
  // weight gradient: rows are the contraction index, so the output tile is free; a group's
  // k range is short (a few slices), which makes the per-tile fixed cost count: large tiles
  if (M >= 256 && N >= 256) {
    p.tiles_m = cdiv(M, 256); p.tiles_n = cdiv(N, 256);
    return launch_k<256, 256, 2, 2, true, true, true, false>(p, st);   // k ranges are whole slices
  }
  return launch_k<128, 128, 2, 2, true, true, true, false>(p, st);
}

}  // namespace bm
