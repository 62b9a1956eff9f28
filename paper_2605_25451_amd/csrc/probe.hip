// Yardstick kernels for the roofline denominators: a register-resident MFMA loop
// (what the matrix cores sustain on this chip at the clock it actually holds under
// load) and a streaming copy (what HBM sustains).  Measuring tools only.
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
