// Shape-agnostic GEMM with fp32 FMA arithmetic.  It is the fp32 check path of
// the block and the cover for shapes the MFMA kernels do not take (tiny or
// oddly sized problems such as the adaLN conditioning projection).
//
//   NT: C[M,N]  = A[M,K] B[N,K]^T      NN: C[M,N] = A[M,K] B[K,N]
//   TN: C[M,N] += A[K,M]^T B[K,N]      (C fp32, accumulated)
//
// 64x64 output tile per workgroup, 16-deep k slices staged in LDS, a 4x4
// register tile per thread.  Every access is bounds-checked.
#include "common.h"

namespace bm {

namespace {

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // k slice

// With k_per_split < K the grid's z index selects a k range and the workgroup stores
// its fp32 partial tile into `partial` [z][M][N]; finish_kernel then sums the ranges
// in order and applies the epilogue (skinny problems: few output tiles, long K).
template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    int M, int N, int K, const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
    void* __restrict__ Cv, int ldc, const T* __restrict__ bias, const T* __restrict__ residual,
    int out_fp32, int k_per_split, float* __restrict__ partial, GemmGroups grp) {
  __shared__ float As[GK][GT + 4];
  __shared__ float Bs[GK][GT + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  int kbeg = blockIdx.z * k_per_split;
  int kfin = min(K, kbeg + k_per_split);
  if (grp.group_rows) {              // grouped weight gradient: blockIdx.z is the group
    kbeg = min(grp.group_rows[blockIdx.z], K);
    kfin = min(grp.group_rows[blockIdx.z + 1], K);
    if (kbeg >= kfin) return;
    Cv = (float*)Cv + (long)blockIdx.z * grp.c_stride;
  } else if (grp.tile_group) {       // grouped forward / input gradient: B of this row block's group
    const int g = grp.tile_group[m0 / MOE_PAD];
    if (g < 0) return;
    B += (long)g * grp.b_stride;
  }
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = kbeg; k0 < kfin; k0 += GK) {
    // A slice -> As[k][m]
    if (LAYOUT == GEMM_TN) {
      int k = tid >> 4, m = (tid & 15) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int gm = m0 + m + e, gk = k0 + k;
        As[k][m + e] = (gm < M && gk < kfin) ? Elt<T>::to_f(A[(size_t)gk * lda + gm]) : 0.f;
      }
    } else {
      int m = tid >> 2, k = (tid & 3) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int gm = m0 + m, gk = k0 + k + e;
        As[k + e][m] = (gm < M && gk < kfin) ? Elt<T>::to_f(A[(size_t)gm * lda + gk]) : 0.f;
      }
    }
    // B slice -> Bs[k][n]
    if (LAYOUT == GEMM_NT) {
      int n = tid >> 2, k = (tid & 3) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int gn = n0 + n, gk = k0 + k + e;
        Bs[k + e][n] = (gn < N && gk < kfin) ? Elt<T>::to_f(B[(size_t)gn * ldb + gk]) : 0.f;
      }
    } else {
      int k = tid >> 4, n = (tid & 15) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int gn = n0 + n + e, gk = k0 + k;
        Bs[k][n + e] = (gn < N && gk < kfin) ? Elt<T>::to_f(B[(size_t)gk * ldb + gn]) : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      size_t idx = (size_t)gm * ldc + gn;
      float v = acc[i][j];
      if (partial) {
        partial[((size_t)blockIdx.z * M + gm) * N + gn] = v;
      } else if (LAYOUT == GEMM_TN) {
        ((float*)Cv)[idx] += v;
      } else {
        if (bias) v += Elt<T>::to_f(bias[gn]);
        if (residual) v += Elt<T>::to_f(residual[idx]);
        if (out_fp32) ((float*)Cv)[idx] = v;
        else ((T*)Cv)[idx] = Elt<T>::from_f(v);
      }
    }
  }
}

template <typename T, int LAYOUT>
__global__ void finish_kernel(const float* __restrict__ partial, int splits, int M, int N,
                              void* __restrict__ Cv, int ldc, const T* __restrict__ bias,
                              const T* __restrict__ residual, int out_fp32) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)M * N) return;
  const int gm = (int)(i / N), gn = (int)(i % N);
  float v = 0.f;
  for (int z = 0; z < splits; ++z) v += partial[(size_t)z * M * N + i];
  const size_t idx = (size_t)gm * ldc + gn;
  if (LAYOUT == GEMM_TN) { ((float*)Cv)[idx] += v; return; }
  if (bias) v += Elt<T>::to_f(bias[gn]);
  if (residual) v += Elt<T>::to_f(residual[idx]);
  if (out_fp32) ((float*)Cv)[idx] = v;
  else ((T*)Cv)[idx] = Elt<T>::from_f(v);
}

int generic_splits(int M, int N, int K) {
  const long tiles = (long)cdiv(M, GT) * cdiv(N, GT);
  if (tiles >= 128 || K < 1024) return 1;
  int s = (int)(512 / tiles);
  const int by_k = K / 128;
  if (s > by_k) s = by_k;
  if (s > 64) s = 64;
  return s < 1 ? 1 : s;
}

template <typename T>
bm_status launch(int layout, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                 void* C, int ldc, const GemmEpilogue& epi, void* scratch, size_t scratch_bytes,
                 hipStream_t st) {
  int splits = generic_splits(M, N, K);
  if ((size_t)splits * M * N * sizeof(float) > scratch_bytes || !scratch) splits = 1;
  const int per = cdiv(cdiv(K, splits), GK) * GK;
  splits = cdiv(K, per);
  float* partial = splits > 1 ? (float*)scratch : nullptr;
  dim3 grid(cdiv(N, GT), cdiv(M, GT), splits), block(256);
#define BM_L(LAY)                                                                               \
  hipLaunchKernelGGL((gemm_generic_kernel<T, LAY>), grid, block, 0, st, M, N, K, (const T*)A,   \
                     lda, (const T*)B, ldb, C, ldc, (const T*)epi.bias, (const T*)epi.residual, \
                     epi.out_fp32, per, partial, GemmGroups{})
  if (layout == GEMM_NT) BM_L(GEMM_NT);
  else if (layout == GEMM_NN) BM_L(GEMM_NN);
  else BM_L(GEMM_TN);
#undef BM_L
  if (partial) {
    const long n = (long)M * N;
#define BM_F(LAY)                                                                               \
  hipLaunchKernelGGL((finish_kernel<T, LAY>), dim3(cdiv(n, 256)), dim3(256), 0, st, partial,    \
                     splits, M, N, C, ldc, (const T*)epi.bias, (const T*)epi.residual, epi.out_fp32)
    if (layout == GEMM_NT) BM_F(GEMM_NT);
    else if (layout == GEMM_NN) BM_F(GEMM_NN);
    else BM_F(GEMM_TN);
#undef BM_F
  }
  BM_CHECK_LAUNCH("gemm_generic");
  return BM_OK;
}

template <typename T>
bm_status launch_grouped(int layout, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                         void* C, int ldc, const GemmGroups& g, hipStream_t st) {
  dim3 grid(cdiv(N, GT), cdiv(M, GT), layout == GEMM_TN ? g.n_groups : 1), block(256);
#define BM_L(LAY)                                                                               \
  hipLaunchKernelGGL((gemm_generic_kernel<T, LAY>), grid, block, 0, st, M, N, K, (const T*)A,   \
                     lda, (const T*)B, ldb, C, ldc, (const T*)nullptr, (const T*)nullptr, 0, K, \
                     (float*)nullptr, g)
  if (layout == GEMM_NT) BM_L(GEMM_NT);
  else if (layout == GEMM_NN) BM_L(GEMM_NN);
  else BM_L(GEMM_TN);
#undef BM_L
  BM_CHECK_LAUNCH("gemm_generic_grouped");
  return BM_OK;
}

}  // namespace

bm_status gemm_generic_grouped(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                               const void* B, int ldb, void* C, int ldc, const GemmGroups& g,
                               hipStream_t st) {
  if (M == 0 || N == 0) return BM_OK;
  GemmGroups gg = g;
  if (layout == GEMM_TN) gg.tile_group = nullptr; else gg.group_rows = nullptr;
  if (dtype == BM_DTYPE_BF16) return launch_grouped<bf16_t>(layout, M, N, K, A, lda, B, ldb, C, ldc, gg, st);
  return launch_grouped<float>(layout, M, N, K, A, lda, B, ldb, C, ldc, gg, st);
}

size_t gemm_generic_scratch_bytes(int M, int N, int K) {
  const int s = generic_splits(M, N, K);
  return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

bm_status gemm_generic(int layout, int dtype, int M, int N, int K, const void* A, int lda,
                       const void* B, int ldb, void* C, int ldc, const GemmEpilogue& epi,
                       void* scratch, size_t scratch_bytes, hipStream_t st) {
  if (M == 0 || N == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    return launch<bf16_t>(layout, M, N, K, A, lda, B, ldb, C, ldc, epi, scratch, scratch_bytes, st);
  return launch<float>(layout, M, N, K, A, lda, B, ldb, C, ldc, epi, scratch, scratch_bytes, st);
}

}  // namespace bm
