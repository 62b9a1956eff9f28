// Yardstick kernels for the roofline denominators: a register-resident MFMA loop
// (what the matrix cores sustain on this chip at the clock it actually holds under
// load) and a streaming copy (what HBM sustains).  Measuring tools only.
#include "common.h"

namespace bm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, long n16) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long)gridDim.x * 256)
    dst[i] = src[i];
}

}  // namespace
}  // namespace bm

using namespace bm;

// Launches `blocks` workgroups of 4 wavefronts, each issuing iters*16 MFMAs of 32x32x16
// (32768 flop per wavefront-MFMA).  The caller times it; flops = blocks*4*iters*16*32768.
extern "C" bm_status bm_probe_mfma(int32_t blocks, int32_t iters, float* out_dev, void* hip_stream) {
  BM_ARG_CHECK(blocks >= 1 && iters >= 1 && out_dev, "bm_probe_mfma: bad arguments");
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, iters, out_dev);
  BM_CHECK_LAUNCH("mfma_probe");
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
