// Module handoff kernels of the micro-unit executor (HBM-bound row moves and the
// stand-in losses): encoder features are scattered into the image-token rows of
// the LLM input and their gradients gathered back (the embed_preprocess step and
// the encoder->LLM / LLM->generator handoffs of Sec. 3.2 "Module handoff", local
// part only -- the cross-rank gather/scatter is out of scope on one GPU).
#include "common.h"

namespace bm {

// dst[rows[i], :] = src[i, :]   (rows distinct)
template <typename T>
__global__ void row_scatter_kernel(const T* __restrict__ src, const int32_t* __restrict__ rows,
                                   T* __restrict__ dst, int n, int width) {
  constexpr int VEC = Elt<T>::VEC;
  const int per = width / VEC;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)n * per) return;
  const int i = (int)(gid / per), c = (int)(gid % per) * VEC;
  *reinterpret_cast<Vec16<T>*>(dst + (size_t)rows[i] * width + c) =
      *reinterpret_cast<const Vec16<T>*>(src + (size_t)i * width + c);
}

// dst[i, :] = src[rows[i], :]
template <typename T>
__global__ void row_gather_kernel(const T* __restrict__ src, const int32_t* __restrict__ rows,
                                  T* __restrict__ dst, int n, int width) {
  constexpr int VEC = Elt<T>::VEC;
  const int per = width / VEC;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)n * per) return;
  const int i = (int)(gid / per), c = (int)(gid % per) * VEC;
  *reinterpret_cast<Vec16<T>*>(dst + (size_t)i * width + c) =
      *reinterpret_cast<const Vec16<T>*>(src + (size_t)rows[i] * width + c);
}

__global__ void fill_zero_kernel(uint4* __restrict__ p, long n16) {
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid < n16) p[gid] = uint4{0u, 0u, 0u, 0u};
}

// a += b (storage dtype, fp32 arithmetic)
template <typename T>
__global__ void add_inplace_kernel(T* __restrict__ a, const T* __restrict__ b, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] = Elt<T>::from_f(Elt<T>::to_f(a[i]) + Elt<T>::to_f(b[i]));
}

// stage 1 of the losses: per-workgroup partial sums in a fixed order
//   MODE 0: grad = (out - target) * inv_n,  partial = 0.5 * inv_n * sum (out - target)^2
//   MODE 1: partial = sum out * target      (grad is `target` itself, not written)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void loss_stage1_kernel(const T* __restrict__ out,
                                                          const T* __restrict__ target,
                                                          T* __restrict__ grad, long n, float inv_n,
                                                          float* __restrict__ partial) {
  __shared__ float sm[4];
  float s = 0.f;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) {
    const float o = Elt<T>::to_f(out[i]), t = Elt<T>::to_f(target[i]);
    if (MODE == 0) {
      const float d = o - t;
      grad[i] = Elt<T>::from_f(d * inv_n);
      s += 0.5f * inv_n * d * d;
    } else {
      s += o * t;
    }
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
}

__global__ void loss_stage2_kernel(const float* __restrict__ partial, int n, float* __restrict__ loss) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < n; ++i) s += partial[i];
    *loss = s;
  }
}

bm_status row_scatter(int dtype, const void* src, const int32_t* rows, void* dst, int n, int width,
                      hipStream_t st) {
  if (n == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  long total = (long)n * (width / vec);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(row_scatter_kernel<bf16_t>, dim3(cdiv(total, 256)), dim3(256), 0, st,
                       (const bf16_t*)src, rows, (bf16_t*)dst, n, width);
  else
    hipLaunchKernelGGL(row_scatter_kernel<float>, dim3(cdiv(total, 256)), dim3(256), 0, st,
                       (const float*)src, rows, (float*)dst, n, width);
  BM_CHECK_LAUNCH("row_scatter");
  return BM_OK;
}

bm_status row_gather(int dtype, const void* src, const int32_t* rows, void* dst, int n, int width,
                     hipStream_t st) {
  if (n == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  long total = (long)n * (width / vec);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(row_gather_kernel<bf16_t>, dim3(cdiv(total, 256)), dim3(256), 0, st,
                       (const bf16_t*)src, rows, (bf16_t*)dst, n, width);
  else
    hipLaunchKernelGGL(row_gather_kernel<float>, dim3(cdiv(total, 256)), dim3(256), 0, st,
                       (const float*)src, rows, (float*)dst, n, width);
  BM_CHECK_LAUNCH("row_gather");
  return BM_OK;
}

bm_status fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return BM_OK;
  long n16 = (long)(bytes / 16);     // buffers here are multiples of 16 bytes
  hipLaunchKernelGGL(fill_zero_kernel, dim3(cdiv(n16, 256)), dim3(256), 0, st, (uint4*)p, n16);
  BM_CHECK_LAUNCH("fill_zero");
  return BM_OK;
}

bm_status add_inplace(int dtype, void* a, const void* b, long n, hipStream_t st) {
  if (n == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(add_inplace_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (bf16_t*)a, (const bf16_t*)b, n);
  else
    hipLaunchKernelGGL(add_inplace_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (float*)a, (const float*)b, n);
  BM_CHECK_LAUNCH("add_inplace");
  return BM_OK;
}

constexpr int LOSS_BLOCKS = 256;
size_t loss_scratch_bytes() { return LOSS_BLOCKS * sizeof(float); }

bm_status mse_loss(int dtype, const void* out, const void* target, void* grad, long n, float* loss,
                   void* scratch, hipStream_t st) {
  const float inv_n = 1.0f / (float)n;
  float* partial = (float*)scratch;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL((loss_stage1_kernel<bf16_t, 0>), dim3(LOSS_BLOCKS), dim3(256), 0, st,
                       (const bf16_t*)out, (const bf16_t*)target, (bf16_t*)grad, n, inv_n, partial);
  else
    hipLaunchKernelGGL((loss_stage1_kernel<float, 0>), dim3(LOSS_BLOCKS), dim3(256), 0, st,
                       (const float*)out, (const float*)target, (float*)grad, n, inv_n, partial);
  hipLaunchKernelGGL(loss_stage2_kernel, dim3(1), dim3(64), 0, st, partial, LOSS_BLOCKS, loss);
  BM_CHECK_LAUNCH("mse_loss");
  return BM_OK;
}

bm_status dot_loss(int dtype, const void* out, const void* g, long n, float* loss, void* scratch,
                   hipStream_t st) {
  float* partial = (float*)scratch;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL((loss_stage1_kernel<bf16_t, 1>), dim3(LOSS_BLOCKS), dim3(256), 0, st,
                       (const bf16_t*)out, (const bf16_t*)g, (bf16_t*)nullptr, n, 0.f, partial);
  else
    hipLaunchKernelGGL((loss_stage1_kernel<float, 1>), dim3(LOSS_BLOCKS), dim3(256), 0, st,
                       (const float*)out, (const float*)g, (float*)nullptr, n, 0.f, partial);
  hipLaunchKernelGGL(loss_stage2_kernel, dim3(1), dim3(64), 0, st, partial, LOSS_BLOCKS, loss);
  BM_CHECK_LAUNCH("dot_loss");
  return BM_OK;
}

}  // namespace bm
