// Yardstick kernels for the roofline denominators: a register-resident MFMA loop
// (what the matrix cores sustain on this chip at the clock it actually holds under
// load), a streaming copy (what HBM sustains), the LDS by instruction kind and the issue
// slots an MFMA leaves to the vector unit.  Measuring tools only.
#include "common.h"

namespace bm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16 independent accumulator blocks per wavefront (the GEMM's register tile), no memory traffic
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* __restrict__ out) {
  f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (bf16_t)(float)(threadIdx.x & 7); b[e] = (bf16_t)(float)(e + 1); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][0];
  if (s == -1.f) out[0] = s;      // keeps the loop alive without writing
}

// The same loop for either MFMA shape and either kind of operand data.  The clock the chip holds
// under matrix load depends on how many operand bits toggle: operands that are all zero keep it at
// its maximum, pseudo-random values of unit scale (what activations look like) lower it, and the
// 16x16x32 shape (a quarter of the accumulator registers written per flop) lowers it less than
// the 32x32x16 shape does.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ inline unsigned probe_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
template <int N>
__device__ inline void probe_operands(bf16x8 (&a)[N], bf16x8 (&b)[N], int random_operands) {
#pragma unroll
  for (int f = 0; f < N; ++f)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float va = 0.f, vb = 0.f;
      if (random_operands) {
        // sum of four uniform bytes, centred and scaled to unit variance: roughly normal
        const unsigned h1 = probe_hash(threadIdx.x * 64 + f * 8 + e + blockIdx.x * 7919u), h2 = probe_hash(h1 + 12345u);
        va = (((h1 & 255) + ((h1 >> 8) & 255) + ((h1 >> 16) & 255) + (h1 >> 24)) / 256.f - 2.f) * 1.73f;
        vb = (((h2 & 255) + ((h2 >> 8) & 255) + ((h2 >> 16) & 255) + (h2 >> 24)) / 256.f - 2.f) * 1.73f;
      }
      a[f][e] = (bf16_t)va; b[f][e] = (bf16_t)vb;
    }
}
template <int SHAPE16>
__global__ __launch_bounds__(256) void mfma_probe_ex_kernel(int iters, int random_operands, float* __restrict__ out) {
  float s = 0.f;
  if (SHAPE16 == 0) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    bf16x8 a[4], b[4];
    probe_operands(a, b, random_operands);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0];
  } else {
    f32x4 acc[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a[8], b[8];
    probe_operands(a, b, random_operands);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 64; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 7], b[i >> 3], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 64; ++i) s += acc[i][0];
  }
  if (s == -1.2345f) out[0] = s;      // keeps the loop alive without writing
}

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, long n16) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long)gridDim.x * 256)
    dst[i] = src[i];
}

// read-only leg: every thread keeps UNROLL 16-byte loads in flight and folds them into one
// word, so nothing is written back (one word per workgroup at the end)
template <int UNROLL>
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4* __restrict__ src, long n16,
                                                         unsigned* __restrict__ out) {
  unsigned acc = 0u;
  const long stride = (long)gridDim.x * 256;
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < n16; i += stride) { const u32x4 v = src[i]; acc ^= v[0] ^ v[1] ^ v[2] ^ v[3]; }
  if (acc == 0x9e3779b9u) out[blockIdx.x & 255] = acc;        // keeps the loads alive
}

// write-only leg
__global__ __launch_bounds__(256) void fill_probe_kernel(u32x4* __restrict__ dst, long n16, unsigned value) {
  const u32x4 v = {value, value, value, value};
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long)gridDim.x * 256)
    __builtin_nontemporal_store(v, dst + i);
}


// LDS throughput by instruction kind, and what an LDS fill costs next to fragment reads (the
// GEMM's and the attention kernels' mix).  Two workgroups of four wavefronts per CU, 64 KiB each,
// conflict-free patterns of a swizzled [rows][128] bf16 tile; nothing leaves the CU except, for
// the direct loads, 16-byte reads of a small buffer that stays in L2.
//   READS : 16 x ds_read_b128 (row fragments) per wavefront and iteration       (16 KiB)
//   TREADS: 16 x 2 ds_read_b64_tr_b16 (transposed fragments)                    (16 KiB)
//   STORES: 8 x ds_write_b128                                                   ( 8 KiB)
//   DIRECT: 8 x global_load_lds_dwordx4                                         ( 8 KiB)
typedef short s16x4 __attribute__((ext_vector_type(4)));
enum : int { LDS_READS = 1, LDS_TREADS = 2, LDS_STORES = 4, LDS_DIRECT = 8 };
template <int WHAT>
__global__ __launch_bounds__(256) void lds_probe_kernel(int iters, const u32x4* __restrict__ g,
                                                        unsigned* __restrict__ out) {
  __shared__ __attribute__((aligned(1024))) u32x4 buf[4096];   // 64 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 4096; i += 256) buf[i] = u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  const int row = lane & 31, half = lane >> 5;
  const int f = ((row & 3) << 2) | ((row >> 2) & 3);
  const int gi = lane >> 4, s16 = lane & 15;
  unsigned acc = 0;
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)buf;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (WHAT & LDS_READS) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const unsigned addr = (wave & 1) * 8192 + row * 256 + ((((j * 2 + h) & 7) * 2 + half) ^ f) * 16 + h * 16384;
          u32x4 v;
          asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
          asm volatile("s_waitcnt lgkmcnt(6)");
          acc += v[0];
        }
      }
      if (WHAT & LDS_TREADS) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int col = (j & 3) * 32 + (gi & 1) * 16 + (s16 & 3) * 4;
          const int r = h * 32 + (j >> 2) * 16 + (gi >> 1) * 4 + (s16 >> 2);
          const int ff = ((r & 3) << 2) | ((r >> 2) & 3);
          const unsigned addr = (wave & 1) * 16384 + r * 256 + (((col >> 3) ^ ff) << 4) + (col & 7) * 2;
          s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(size_t)addr);
          s16x4 w = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(size_t)(addr + 2048));
          acc += v[0] + w[0];
        }
      }
      if (WHAT & LDS_STORES) {
        const unsigned addr = 32768 + ((wave * 8 + j) & 31) * 1024 + lane * 16;
        const u32x4 v = {(unsigned)it, 0u, 0u, 0u};
        asm volatile("ds_write_b128 %0, %1" :: "v"(addr), "v"(v));
      }
      if (WHAT & LDS_DIRECT) {
        const unsigned dst = lds0 + 32768 + ((wave * 8 + j) & 31) * 1024;
        const unsigned voff = (((blockIdx.x & 7) * 64 + ((wave * 8 + j + it) & 63)) * 64 + lane) * 16;   // < 512 KiB
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(dst), "v"(voff), "s"(g) : "memory", "m0");
      }
    }
    if (WHAT & LDS_DIRECT) asm volatile("s_waitcnt vmcnt(0)");
  }
  asm volatile("s_waitcnt lgkmcnt(0)");
  if (acc == 0x12345678u) out[0] = acc;      // keeps the reads alive without writing
}

// One wavefront per SIMD: groups of one 32x32x16 MFMA followed by NV independent vector
// instructions.  The matrix pipe takes an MFMA every 32 clocks; what the group takes beyond that
// is vector issue time that did not fit beside the MFMA.
template <int NV>
__global__ __launch_bounds__(256) void issue_probe_kernel(int iters, float* __restrict__ out) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (bf16_t)0.f; b[e] = (bf16_t)0.f; }
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 0.f;
  const float c1 = 0.5f, c2 = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[gq]) : "v"(a), "v"(b));
#pragma unroll
      for (int i = 0; i < NV; ++i) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i & 7]) : "v"(c1), "v"(c2));
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += acc[i][0];
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
  if (s == -1.2345f) out[0] = s;
}

}  // namespace
}  // namespace bm

using namespace bm;

// Read-only and write-only legs of the HBM yardstick: bm_probe_read streams bytes (multiple of 16)
// from src with `blocks` workgroups of 256 threads, each thread holding `unroll` (1, 4 or 8)
// 16-byte loads in flight; bm_probe_fill writes bytes to dst.  out_dev: 256 words (dev).
extern "C" bm_status bm_probe_read(const void* src, size_t bytes, int32_t blocks, int32_t unroll,
                                   void* out_dev, void* hip_stream) {
  BM_ARG_CHECK(src && out_dev && bytes % 16 == 0 && blocks >= 1, "bm_probe_read: bad arguments");
  BM_ARG_CHECK(unroll == 1 || unroll == 4 || unroll == 8, "bm_probe_read: unroll must be 1, 4 or 8");
  const long n16 = (long)(bytes / 16);
  hipStream_t st = (hipStream_t)hip_stream;
  if (unroll == 1) hipLaunchKernelGGL(read_probe_kernel<1>, dim3(blocks), dim3(256), 0, st, (const u32x4*)src, n16, (unsigned*)out_dev);
  else if (unroll == 4) hipLaunchKernelGGL(read_probe_kernel<4>, dim3(blocks), dim3(256), 0, st, (const u32x4*)src, n16, (unsigned*)out_dev);
  else hipLaunchKernelGGL(read_probe_kernel<8>, dim3(blocks), dim3(256), 0, st, (const u32x4*)src, n16, (unsigned*)out_dev);
  BM_CHECK_LAUNCH("read_probe");
  return BM_OK;
}

extern "C" bm_status bm_probe_fill(void* dst, size_t bytes, int32_t blocks, void* hip_stream) {
  BM_ARG_CHECK(dst && bytes % 16 == 0 && blocks >= 1, "bm_probe_fill: bad arguments");
  hipLaunchKernelGGL(fill_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, (u32x4*)dst,
                     (long)(bytes / 16), 0x3f803f80u);
  BM_CHECK_LAUNCH("fill_probe");
  return BM_OK;
}

// Launches `blocks` workgroups of 4 wavefronts, each issuing iters*16 MFMAs of 32x32x16
// (32768 flop per wavefront-MFMA).  The caller times it; flops = blocks*4*iters*16*32768.
extern "C" bm_status bm_probe_mfma(int32_t blocks, int32_t iters, float* out_dev, void* hip_stream) {
  BM_ARG_CHECK(blocks >= 1 && iters >= 1 && out_dev, "bm_probe_mfma: bad arguments");
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, iters, out_dev);
  BM_CHECK_LAUNCH("mfma_probe");
  return BM_OK;
}

// bm_probe_mfma with a choice of MFMA shape (shape16 = 0: 32x32x16, 16 per iteration; 1: 16x16x32,
// 64 per iteration) and of operand data (random_operands = 0: zeros, 1: pseudo-random values of unit
// scale).  flops = blocks * 4 * iters * 2^19 (shape16 = 0) or 2^20 (shape16 = 1).
extern "C" bm_status bm_probe_mfma_ex(int32_t blocks, int32_t iters, int32_t shape16, int32_t random_operands,
                                      float* out_dev, void* hip_stream) {
  BM_ARG_CHECK(blocks >= 1 && iters >= 1 && out_dev, "bm_probe_mfma_ex: bad arguments");
  BM_ARG_CHECK((shape16 == 0 || shape16 == 1) && (random_operands == 0 || random_operands == 1),
               "bm_probe_mfma_ex: shape16 and random_operands are 0 or 1");
  if (shape16) hipLaunchKernelGGL(mfma_probe_ex_kernel<1>, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, iters, random_operands, out_dev);
  else hipLaunchKernelGGL(mfma_probe_ex_kernel<0>, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, iters, random_operands, out_dev);
  BM_CHECK_LAUNCH("mfma_probe_ex");
  return BM_OK;
}

// dst[0..bytes) = src[0..bytes), bytes a multiple of 16; moves 2*bytes through HBM.
extern "C" bm_status bm_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  BM_ARG_CHECK(src && dst && bytes % 16 == 0, "bm_probe_copy: bad arguments");
  hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint4*)src, (uint4*)dst, (long)(bytes / 16));
  BM_CHECK_LAUNCH("copy_probe");
  return BM_OK;
}

// LDS yardstick: launches 512 workgroups (two per CU) of 4 wavefronts; per wavefront and iteration
// `what` (a sum of 1: 16 KiB of row-fragment reads, 2: 16 KiB of transposed-fragment reads,
// 4: 8 KiB of LDS stores, 8: 8 KiB of direct-to-LDS loads from src_dev) moves through the LDS.
// Supported sums: 1, 2, 4, 8, 5 (reads next to stores), 9 (reads next to direct loads).
// src_dev: at least 512 KiB (dev), read only by the direct loads; out_dev: one word (dev).
extern "C" bm_status bm_probe_lds(int32_t what, int32_t iters, const void* src_dev, size_t src_bytes,
                                  void* out_dev, void* hip_stream) {
  BM_ARG_CHECK(iters >= 1 && out_dev, "bm_probe_lds: bad arguments");
  BM_ARG_CHECK(what == 1 || what == 2 || what == 4 || what == 8 || what == 5 || what == 9,
               "bm_probe_lds: what must be 1, 2, 4, 8, 5 or 9");
  BM_ARG_CHECK(!(what & 8) || (src_dev && src_bytes >= (size_t)512 * 1024),
               "bm_probe_lds: the direct loads read 512 KiB of src_dev");
  hipStream_t st = (hipStream_t)hip_stream;
  const u32x4* g = (const u32x4*)src_dev;
  unsigned* o = (unsigned*)out_dev;
#define BM_L(W) hipLaunchKernelGGL(lds_probe_kernel<W>, dim3(512), dim3(256), 0, st, iters, g, o)
  switch (what) {
    case 1: BM_L(1); break;
    case 2: BM_L(2); break;
    case 4: BM_L(4); break;
    case 8: BM_L(8); break;
    case 5: BM_L(5); break;
    default: BM_L(9); break;
  }
#undef BM_L
  BM_CHECK_LAUNCH("lds_probe");
  return BM_OK;
}

// Issue yardstick: 256 workgroups of 4 wavefronts (one per SIMD), iters x 4 groups of one
// 32x32x16 MFMA and n_valu (0, 4 or 8) independent vector instructions each.  out_dev: one float (dev).
extern "C" bm_status bm_probe_issue(int32_t n_valu, int32_t iters, float* out_dev, void* hip_stream) {
  BM_ARG_CHECK(iters >= 1 && out_dev, "bm_probe_issue: bad arguments");
  BM_ARG_CHECK(n_valu == 0 || n_valu == 4 || n_valu == 8, "bm_probe_issue: n_valu must be 0, 4 or 8");
  hipStream_t st = (hipStream_t)hip_stream;
  if (n_valu == 0) hipLaunchKernelGGL(issue_probe_kernel<0>, dim3(256), dim3(256), 0, st, iters, out_dev);
  else if (n_valu == 4) hipLaunchKernelGGL(issue_probe_kernel<4>, dim3(256), dim3(256), 0, st, iters, out_dev);
  else hipLaunchKernelGGL(issue_probe_kernel<8>, dim3(256), dim3(256), 0, st, iters, out_dev);
  BM_CHECK_LAUNCH("issue_probe");
  return BM_OK;
}
