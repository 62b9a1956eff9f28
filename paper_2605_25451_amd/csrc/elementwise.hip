// HBM-bound kernels of the block: norms (LayerNorm / RMSNorm / affine-free LN
// with adaLN modulation) forward and backward, RoPE, GELU / SwiGLU, column and
// per-sequence reductions for bias / gamma / adaLN gradients.
//
// Access pattern: every kernel moves 16 bytes per lane per access, with a
// wavefront covering one contiguous 1 KiB span of a row, and reduces inside a
// wavefront with cross-lane shuffles (no LDS, no barrier, on the per-row
// paths).  Arithmetic is fp32 whatever the storage type.
#include "common.h"

namespace bm {

// ------------------------------------------------------------------ tok_seq
__global__ void tok_seq_kernel(const int32_t* __restrict__ cu, int S, int T,
                               int32_t* __restrict__ tok_seq) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  int lo = 0, hi = S;   // find s with cu[s] <= t < cu[s+1]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  tok_seq[t] = lo;
}

bm_status launch_tok_seq(const int32_t* cu_dev, int S, int T, int32_t* tok_seq, hipStream_t st) {
  hipLaunchKernelGGL(tok_seq_kernel, dim3(cdiv(T, 256)), dim3(256), 0, st, cu_dev, S, T, tok_seq);
  BM_CHECK_LAUNCH("tok_seq");
  return BM_OK;
}

// ------------------------------------------------------------------ norm forward
// One wavefront per row; the row lives in registers (NV 16-byte vectors per lane).
template <typename T, int KIND, int NV>
__global__ __launch_bounds__(256) void norm_fwd_kernel(
    const T* __restrict__ x, T* __restrict__ h, float* __restrict__ stats,
    const T* __restrict__ gamma, const T* __restrict__ beta, const float* __restrict__ mod,
    int ld_mod, int shift_off, int scale_off, const int32_t* __restrict__ tok_seq, int rows, int d,
    float eps, int write_stats) {
  constexpr int VEC = Elt<T>::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * d;
  float buf[NV][VEC];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int col = (i * WAVE + lane) * VEC;
    if (col < d) {
      load16(xr + col, buf[i]);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) buf[i][e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) s += (KIND == BM_NORM_RMSNORM) ? buf[i][e] * buf[i][e] : buf[i][e];
  }
  s = wave_sum(s);
  float mean = 0.f, rstd;
  const float inv_d = 1.0f / (float)d;
  if (KIND == BM_NORM_RMSNORM) {
    rstd = 1.0f / sqrtf(s * inv_d + eps);
  } else {
    mean = s * inv_d;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int col = (i * WAVE + lane) * VEC;
      if (col < d) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { float c = buf[i][e] - mean; v += c * c; }
      }
    }
    v = wave_sum(v);
    rstd = 1.0f / sqrtf(v * inv_d + eps);
  }
  if (write_stats && lane == 0) { stats[row] = mean; stats[rows + row] = rstd; }
  T* hr = h + (size_t)row * d;
  const float* mrow = nullptr;
  if (KIND == BM_NORM_ADALN) mrow = mod + (size_t)tok_seq[row] * ld_mod;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int col = (i * WAVE + lane) * VEC;
    if (col >= d) continue;
    float out[VEC];
    if (KIND == BM_NORM_LAYERNORM) {
      float g[VEC], b[VEC];
      load16(gamma + col, g); load16(beta + col, b);
#pragma unroll
      for (int e = 0; e < VEC; ++e) out[e] = (buf[i][e] - mean) * rstd * g[e] + b[e];
    } else if (KIND == BM_NORM_RMSNORM) {
      float g[VEC];
      load16(gamma + col, g);
#pragma unroll
      for (int e = 0; e < VEC; ++e) out[e] = buf[i][e] * rstd * g[e];
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        out[e] = (buf[i][e] - mean) * rstd * (1.0f + mrow[scale_off + col + e]) + mrow[shift_off + col + e];
    }
    store16(hr + col, out);
  }
}

template <typename T, int KIND>
static bm_status norm_fwd_dispatch(const NormArgs& a, const void* x, void* h, float* stats,
                                   int write_stats, hipStream_t st) {
  constexpr int VEC = Elt<T>::VEC;
  int nv = cdiv(a.d, WAVE * VEC);
  dim3 grid(cdiv(a.T, 4)), block(256);
#define BM_LAUNCH_NV(NVV)                                                                        \
  hipLaunchKernelGGL((norm_fwd_kernel<T, KIND, NVV>), grid, block, 0, st, (const T*)x, (T*)h,    \
                     stats, (const T*)a.gamma, (const T*)a.beta, a.mod, a.ld_mod, a.shift_off,   \
                     a.scale_off, a.tok_seq, a.T, a.d, a.eps, write_stats)
  if (nv <= 1) BM_LAUNCH_NV(1);
  else if (nv <= 2) BM_LAUNCH_NV(2);
  else if (nv <= 4) BM_LAUNCH_NV(4);
  else if (nv <= 8) BM_LAUNCH_NV(8);
  else if (nv <= 16) BM_LAUNCH_NV(16);
  else { set_error("norm: hidden %d too wide", a.d); return BM_ERR_UNSUPPORTED; }
#undef BM_LAUNCH_NV
  BM_CHECK_LAUNCH("norm_fwd");
  return BM_OK;
}

bm_status norm_forward(const NormArgs& a, const void* x, void* h, float* stats, int write_stats,
                       hipStream_t st) {
  if (a.T == 0) return BM_OK;
#define BM_KIND(TT)                                                                              \
  switch (a.kind) {                                                                              \
    case BM_NORM_LAYERNORM: return norm_fwd_dispatch<TT, BM_NORM_LAYERNORM>(a, x, h, stats, write_stats, st); \
    case BM_NORM_RMSNORM: return norm_fwd_dispatch<TT, BM_NORM_RMSNORM>(a, x, h, stats, write_stats, st);     \
    default: return norm_fwd_dispatch<TT, BM_NORM_ADALN>(a, x, h, stats, write_stats, st);       \
  }
  if (a.dtype == BM_DTYPE_BF16) { BM_KIND(bf16_t) } else { BM_KIND(float) }
#undef BM_KIND
}

// ------------------------------------------------------------------ norm backward
// Each wavefront walks rows with a grid stride; every lane owns the same
// columns on every row, so column sums accumulate in registers and leave the
// kernel as NP partial rows per workgroup: gamma (and beta) gradients, and with
// SUMS also the column sums of the residual gradient read here and of the
// gradient written here (the bias gradients of the two neighbouring linear
// layers, whose output gradients these are).  With h_out the normalised row is
// written again for the weight-gradient GEMM that follows.
// (grid cap: every workgroup ends with a fixed-order combine of its wavefronts and leaves NP
// partial rows, so narrow rows want few workgroups; wide rows, whose wavefronts hold many registers,
// want more of them in flight)
constexpr int NORM_BWD_MAX_BLOCKS = 768, NORM_BWD_MAX_BLOCKS_WIDE = 1024;

template <int KIND, bool SUMS> struct NormBwdParts {
  static constexpr int NP = (KIND == BM_NORM_LAYERNORM ? 2 : KIND == BM_NORM_RMSNORM ? 1 : 0) + (SUMS ? 2 : 0);
};

// wavefronts per workgroup (eight were measured slower: 512 threads cap the registers
// per lane at 128 and the column accumulators spill)
template <int NV> struct NormBwdWaves { static constexpr int N = 4; };

// SPLIT wavefronts share one row (wide rows: half the registers per wavefront, twice the resident
// wavefronts); they exchange their partial row sums through LDS, one barrier per row.
template <typename T, int KIND, int NV, bool SUMS, int SPLIT = 1>
__global__ __launch_bounds__(NormBwdWaves<NV>::N * 64) void norm_bwd_kernel(
    const T* __restrict__ x, const float* __restrict__ stats, const T* __restrict__ dh,
    const T* __restrict__ dres, T* __restrict__ dx, T* __restrict__ h_out,
    const T* __restrict__ gamma, const T* __restrict__ beta,
    const float* __restrict__ mod, int ld_mod, int shift_off, int scale_off,
    const int32_t* __restrict__ tok_seq, float* __restrict__ partial /* [gridDim.x][NP][d] */,
    int rows, int d) {
  constexpr int VEC = Elt<T>::VEC;
  constexpr int NP = NormBwdParts<KIND, SUMS>::NP;
  constexpr int NS = SUMS ? NV : 1;
  constexpr int NW = NormBwdWaves<NV>::N;
  constexpr int RPB = NW / SPLIT;          // rows per workgroup and trip
  extern __shared__ float sm[];   // [d]
  __shared__ float rowsum[2][RPB][SPLIT][2];     // two trips' worth: one barrier per trip is enough
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int slot = wave / SPLIT, part = wave % SPLIT;
  // column of vector i of this wavefront
  auto col_of = [&](int i) { return ((i * SPLIT + part) * WAVE + lane) * VEC; };
  float gam[NV][VEC];
  float acc_g[NV][VEC], acc_b[NV][VEC];
  float acc_r[NS][VEC], acc_o[NS][VEC];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int col = col_of(i);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc_g[i][e] = 0.f; acc_b[i][e] = 0.f; gam[i][e] = 1.f; }
    if (KIND != BM_NORM_ADALN && col < d) load16(gamma + col, gam[i]);
  }
#pragma unroll
  for (int i = 0; i < NS; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc_r[i][e] = 0.f; acc_o[i][e] = 0.f; }
  const float inv_d = 1.0f / (float)d;
  int trip = 0;
  // With rows shared between wavefronts every wavefront of the workgroup makes the same trips (the
  // barrier below); one whose row lies past the end works on the last row again and stores nothing.
  // Unshared rows need neither: such a wavefront simply stops.
  for (int base = blockIdx.x * RPB; SPLIT > 1 ? base < rows : base + slot < rows; base += gridDim.x * RPB, ++trip) {
    const bool live = SPLIT > 1 ? base + slot < rows : true;
    const int row = live ? base + slot : rows - 1;
    const size_t off = (size_t)row * d;
    const float mean = stats[row], rstd = stats[rows + row];
    const float* mrow = nullptr;
    if (KIND == BM_NORM_ADALN) mrow = mod + (size_t)tok_seq[row] * ld_mod;
    // The residual gradient is only needed after the row reductions.  Narrow rows fetch it with
    // the rest (one memory latency per row less); wide rows would pay for that with registers
    // and lose a resident wavefront, so they fetch it late.
    constexpr bool EARLY_RES = NV <= 4;
    float xv[NV][VEC], gv[NV][VEC], resv[EARLY_RES ? NV : 1][VEC];
    float s1 = 0.f, s2 = 0.f;
    if (EARLY_RES) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int col = col_of(i);
        if (col < d) load16(dres + off + col, resv[EARLY_RES ? i : 0]);
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int col = col_of(i);
      if (col < d) {
        float dhv[VEC];
        load16(x + off + col, xv[i]);
        load16(dh + off + col, dhv);
        if (!live) {          // a repeated row must not count in the column sums
#pragma unroll
          for (int e = 0; e < VEC; ++e) dhv[e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float g;
          if (KIND == BM_NORM_ADALN) g = dhv[e] * (1.0f + mrow[scale_off + col + e]);
          else g = dhv[e] * gam[i][e];
          if (KIND == BM_NORM_RMSNORM) {
            s2 += g * xv[i][e];
            acc_g[i][e] += dhv[e] * xv[i][e] * rstd;
          } else {
            float xh = (xv[i][e] - mean) * rstd;
            xv[i][e] = xh;
            s1 += g; s2 += g * xh;
            acc_g[i][e] += dhv[e] * xh;
            acc_b[i][e] += dhv[e];
          }
          gv[i][e] = g;
        }
      }
    }
    s2 = wave_sum(s2);
    if (KIND != BM_NORM_RMSNORM) s1 = wave_sum(s1);
    if (SPLIT > 1) {
      if (lane == 0) { rowsum[trip & 1][slot][part][0] = s1; rowsum[trip & 1][slot][part][1] = s2; }
      __syncthreads();
      s1 = 0.f; s2 = 0.f;
#pragma unroll
      for (int q = 0; q < SPLIT; ++q) { s1 += rowsum[trip & 1][slot][q][0]; s2 += rowsum[trip & 1][slot][q][1]; }
    }
    s2 *= inv_d;
    s1 *= inv_d;
    const float r3 = rstd * rstd * rstd;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int col = col_of(i);
      if (col < d) {
        float out[VEC], res[VEC];
        if (EARLY_RES) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) res[e] = resv[EARLY_RES ? i : 0][e];
        } else {
          load16(dres + off + col, res);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float v;
          if (KIND == BM_NORM_RMSNORM) v = rstd * gv[i][e] - xv[i][e] * r3 * s2;
          else v = rstd * (gv[i][e] - s1 - xv[i][e] * s2);
          out[e] = res[e] + v;
        }
        if (live) store16(dx + off + col, out);
        if (SUMS) {
          // sum what the consumer reads: the stored (rounded) gradient
          float stored[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) stored[e] = Elt<T>::to_f(Elt<T>::from_f(out[e]));
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            acc_r[SUMS ? i : 0][e] += live ? res[e] : 0.f;
            acc_o[SUMS ? i : 0][e] += live ? stored[e] : 0.f;
          }
        }
        if (h_out) {
          float hv[VEC];
          if (KIND == BM_NORM_LAYERNORM) {
            float bt[VEC];
            load16(beta + col, bt);
#pragma unroll
            for (int e = 0; e < VEC; ++e) hv[e] = xv[i][e] * gam[i][e] + bt[e];
          } else if (KIND == BM_NORM_RMSNORM) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) hv[e] = xv[i][e] * rstd * gam[i][e];
          } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e)
              hv[e] = xv[i][e] * (1.0f + mrow[scale_off + col + e]) + mrow[shift_off + col + e];
          }
          if (live) store16(h_out + off + col, hv);
        }
      }
    }
  }
  // combine the wavefronts through LDS, one after the other (fixed order);
  // adaLN shift/scale gradients are per-sequence sums and have their own kernel
  for (int which = 0; which < NP; ++which) {
    const int what = KIND == BM_NORM_ADALN ? which + 2 : (KIND == BM_NORM_RMSNORM && which > 0 ? which + 1 : which);
    for (int w = 0; w < NW; ++w) {
      if (wave == w) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int col = col_of(i);
          if (col < d) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              float v = what == 0 ? acc_g[i][e] : what == 1 ? acc_b[i][e]
                      : what == 2 ? acc_r[SUMS ? i : 0][e] : acc_o[SUMS ? i : 0][e];
              if (w < SPLIT) sm[col + e] = v; else sm[col + e] += v;   // the first wavefront on these columns
            }
          }
        }
      }
      __syncthreads();
    }
    float* prow = partial + ((size_t)blockIdx.x * NP + which) * d;
    for (int c = threadIdx.x; c < d; c += NW * 64) prow[c] = sm[c];
    __syncthreads();
  }
}

// out[c] += sum over parts of partial[p*stride + c]; 64 columns per workgroup,
// sixteen groups of parts combined through LDS in a fixed order.
constexpr int PR_GROUPS = 16;
__global__ __launch_bounds__(64 * PR_GROUPS) void partial_reduce_kernel(
    const float* __restrict__ partial, int nparts, int stride, int n, float* __restrict__ out) {
  __shared__ float sm[PR_GROUPS][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int g = threadIdx.x >> 6;
  // eight independent loads in flight per thread: the partials come from L2 or further away and
  // the loop is bound by that latency, not by bandwidth
  float s[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) s[u] = 0.f;
  if (c < n) {
    int p = g;
    for (; p + 7 * PR_GROUPS < nparts; p += 8 * PR_GROUPS) {
#pragma unroll
      for (int u = 0; u < 8; ++u) s[u] += partial[(size_t)(p + u * PR_GROUPS) * stride + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p + u * PR_GROUPS < nparts) s[u] += partial[(size_t)(p + u * PR_GROUPS) * stride + c];
  }
  sm[g][threadIdx.x & 63] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  if (g == 0 && c < n) {
    const int l = threadIdx.x;
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < PR_GROUPS; ++i) t += sm[i][l];
    out[c] += t;
  }
}

// The same reduction for up to four destinations in one launch (blockIdx.y
// selects one); they share nparts, stride and n.
struct ReduceTargets { const float* partial[4]; float* out[4]; };
__global__ __launch_bounds__(64 * PR_GROUPS) void partial_reduce_multi_kernel(
    ReduceTargets t, int nparts, int stride, int n) {
  __shared__ float sm[PR_GROUPS][64];
  const float* __restrict__ partial = t.partial[blockIdx.y];
  float* __restrict__ out = t.out[blockIdx.y];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int g = threadIdx.x >> 6;
  // eight independent loads in flight per thread: the partials come from L2 or further away and
  // the loop is bound by that latency, not by bandwidth
  float s[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) s[u] = 0.f;
  if (c < n) {
    int p = g;
    for (; p + 7 * PR_GROUPS < nparts; p += 8 * PR_GROUPS) {
#pragma unroll
      for (int u = 0; u < 8; ++u) s[u] += partial[(size_t)(p + u * PR_GROUPS) * stride + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p + u * PR_GROUPS < nparts) s[u] += partial[(size_t)(p + u * PR_GROUPS) * stride + c];
  }
  sm[g][threadIdx.x & 63] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  if (g == 0 && c < n) {
    const int l = threadIdx.x;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < PR_GROUPS; ++i) v += sm[i][l];
    out[c] += v;
  }
}

// ------------------------------------------------------------------ per-sequence column sums
// Sums over the rows of every sequence, for the adaLN parameter gradients.  A workgroup owns one
// part (of `parts`) of one sequence's rows and 64 16-byte column chunks; its four wavefronts take
// rows round-robin, are combined through LDS in a fixed order, and the parts of a sequence are
// added in a fixed order by seg_reduce_kernel (parts == 1 writes the result directly).
//   MODE 0 (gate):   sum0[s] = sum_t a*b;  optionally gated[t] = a[t] * gate[s]
//   MODE 1 (adaLN):  sum0[s] = sum_t dh,  sum1[s] = sum_t dh * xhat   (xhat from x and the row statistics)
struct SegArgs {
  const void *a, *b;              // MODE 0: a, b.  MODE 1: dh, x
  const float* stats;             // MODE 1: mean[rows], rstd[rows]
  const float* gate; int ld_gate; // MODE 0: gate[s, :] (fp32), used when gated != nullptr
  void* gated;
  const int32_t* cu;
  float* out; int ld_out, off0, off1;   // out[s, off_p + n]
  float* partial;                 // [S*parts][planes][N] when parts > 1
  int parts, rows, N;
};

template <typename T, int MODE>
__global__ __launch_bounds__(256) void seg_sums_kernel(SegArgs p) {
  constexpr int VEC = Elt<T>::VEC;
  constexpr int P = MODE == 0 ? 1 : 2;
  __shared__ float sm[P][4][WAVE * VEC];
  const int s = blockIdx.x / p.parts, part = blockIdx.x % p.parts;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = (blockIdx.y * WAVE + lane) * VEC;
  const bool live = col < p.N;
  const int t0 = p.cu[s], t1 = p.cu[s + 1];
  const int per = (t1 - t0 + p.parts - 1) / p.parts;
  const int rb = t0 + part * per, re = min(t1, rb + per);
  const T* a = (const T*)p.a;
  const T* b = (const T*)p.b;
  float acc[P][VEC], g[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { acc[0][e] = 0.f; acc[P - 1][e] = 0.f; g[e] = 0.f; }
  if (MODE == 0 && p.gated && live) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) g[e] = p.gate[(size_t)s * p.ld_gate + col + e];
  }
  if (live) {
    for (int t = rb + wave; t < re; t += 4) {
      float va[VEC], vb[VEC];
      load16(a + (size_t)t * p.N + col, va);
      load16(b + (size_t)t * p.N + col, vb);
      if (MODE == 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[0][e] += va[e] * vb[e];
        if (p.gated) {
          float o[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) o[e] = va[e] * g[e];
          store16((T*)p.gated + (size_t)t * p.N + col, o);
        }
      } else {
        const float mean = p.stats[t], rstd = p.stats[p.rows + t];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc[0][e] += va[e];
          acc[P - 1][e] += va[e] * ((vb[e] - mean) * rstd);
        }
      }
    }
  }
#pragma unroll
  for (int q = 0; q < P; ++q)
#pragma unroll
    for (int e = 0; e < VEC; ++e) sm[q][wave][lane * VEC + e] = acc[q][e];
  __syncthreads();
  if (wave == 0 && live) {
#pragma unroll
    for (int q = 0; q < P; ++q) {
      float* dst = p.parts > 1 ? p.partial + ((size_t)blockIdx.x * P + q) * p.N + col
                               : p.out + (size_t)s * p.ld_out + (q == 0 ? p.off0 : p.off1) + col;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int c = lane * VEC + e;
        dst[e] = sm[q][0][c] + sm[q][1][c] + sm[q][2][c] + sm[q][3][c];
      }
    }
  }
}

__global__ void seg_reduce_kernel(const float* __restrict__ partial, int S, int parts, int planes, int N,
                                  float* __restrict__ out, int ld_out, int off0, int off1) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)S * planes * N) return;
  const int n = (int)(i % N), q = (int)((i / N) % planes), s = (int)(i / ((long)N * planes));
  float v = 0.f;
  for (int r = 0; r < parts; ++r) v += partial[(((size_t)s * parts + r) * planes + q) * N + n];
  out[(size_t)s * ld_out + (q == 0 ? off0 : off1) + n] = v;
}

// parts per sequence: enough workgroups to fill the chip, at most 16
static int seg_parts(int S, int N, int vec) {
  const long blocks = (long)S * cdiv(N, WAVE * vec);
  if (blocks >= 1024) return 1;
  const int r = cdiv(1024, blocks);
  return r > 16 ? 16 : r;
}

// upper bound for any S: parts > 1 only while S * column blocks < 1024, and then
// S * parts * N <= 2048 * 64 * VEC elements per plane
size_t segment_scratch_bytes() { return (size_t)2048 * 512 * 2 * sizeof(float); }

template <int MODE>
static bm_status seg_launch(int dtype, SegArgs p, int S, void* scratch, hipStream_t st) {
  if (S == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (p.N % vec) { set_error("segment sums: width %d not a multiple of %d", p.N, vec); return BM_ERR_UNSUPPORTED; }
  p.parts = scratch ? seg_parts(S, p.N, vec) : 1;
  p.partial = (float*)scratch;
  dim3 grid(S * p.parts, cdiv(p.N, WAVE * vec));
  if (dtype == BM_DTYPE_BF16) hipLaunchKernelGGL((seg_sums_kernel<bf16_t, MODE>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((seg_sums_kernel<float, MODE>), grid, dim3(256), 0, st, p);
  if (p.parts > 1) {
    const int planes = MODE == 0 ? 1 : 2;
    hipLaunchKernelGGL(seg_reduce_kernel, dim3(cdiv((long)S * planes * p.N, 256)), dim3(256), 0, st, p.partial, S,
                       p.parts, planes, p.N, p.out, p.ld_out, p.off0, p.off1);
  }
  BM_CHECK_LAUNCH("segment sums");
  return BM_OK;
}

bm_status segment_gate(int dtype, const void* a, const void* b, const float* gate, int ld_gate, void* gated,
                       const int32_t* cu_dev, int S, int N, float* out, int ld_out, void* scratch,
                       hipStream_t st) {
  SegArgs p{};
  p.a = a; p.b = b; p.gate = gate; p.ld_gate = ld_gate; p.gated = gated; p.cu = cu_dev;
  p.out = out; p.ld_out = ld_out; p.off0 = 0; p.off1 = 0; p.N = N;
  return seg_launch<0>(dtype, p, S, scratch, st);
}

static int norm_bwd_blocks(int T, int d) {
  const int cap = d >= 2048 ? NORM_BWD_MAX_BLOCKS_WIDE : NORM_BWD_MAX_BLOCKS;
  const int b = cdiv(T, 4);
  return b < cap ? b : cap;
}

size_t norm_backward_scratch_bytes(int T, int d) {
  return align_up((size_t)norm_bwd_blocks(T, d) * 4 * d * sizeof(float), 256) + segment_scratch_bytes();
}

template <typename T, int KIND, bool SUMS>
static bm_status norm_bwd_dispatch(const NormArgs& a, const void* x, const float* stats,
                                   const void* dh, const void* dres, void* dx, void* h_out,
                                   float* partial, hipStream_t st) {
  constexpr int VEC = Elt<T>::VEC;
  int nv = cdiv(a.d, WAVE * VEC);
  dim3 grid(norm_bwd_blocks(a.T, a.d));
  size_t lds = (size_t)a.d * sizeof(float);
#define BM_LAUNCH_NV(NVV, SP)                                                                    \
  hipLaunchKernelGGL((norm_bwd_kernel<T, KIND, NVV, SUMS, SP>), grid, dim3(NormBwdWaves<NVV>::N * 64), lds, st, (const T*)x,   \
                     stats, (const T*)dh, (const T*)dres, (T*)dx, (T*)h_out, (const T*)a.gamma,  \
                     (const T*)a.beta, a.mod, a.ld_mod, a.shift_off, a.scale_off, a.tok_seq,     \
                     partial, a.T, a.d)
  // rows of 4 or more vectors per lane are shared by two wavefronts (measured: 1152-wide rows are
  // faster unshared, 2048-wide and wider ones shared)
  if (nv <= 1) BM_LAUNCH_NV(1, 1);
  else if (nv <= 2) { if (SUMS) BM_LAUNCH_NV(1, 2); else BM_LAUNCH_NV(2, 1); }
  else if (nv <= 3) BM_LAUNCH_NV(4, 1);
  else if (nv <= 4) BM_LAUNCH_NV(2, 2);
  else if (nv <= 8) BM_LAUNCH_NV(4, 2);
  else if (nv <= 16) BM_LAUNCH_NV(8, 2);
  else { set_error("norm: hidden %d too wide", a.d); return BM_ERR_UNSUPPORTED; }
#undef BM_LAUNCH_NV
  BM_CHECK_LAUNCH("norm_bwd");
  return BM_OK;
}

// dsum_res / dsum_out (both or neither): fp32 vectors that receive += the column
// sums of dres and of dx.
bm_status norm_backward(const NormArgs& a, const void* x, const float* stats, const void* dh,
                        const void* dres, void* dx, void* h_out, float* dgamma, float* dbeta,
                        float* dsum_res, float* dsum_out, float* dmod, const int32_t* cu_dev, int S,
                        void* scratch, hipStream_t st) {
  if (a.T == 0) return BM_OK;
  float* partial = (float*)scratch;
  const bool sums = dsum_res != nullptr;
  if (sums != (dsum_out != nullptr)) { set_error("norm_backward: one column-sum target without the other"); return BM_ERR_INVALID_ARG; }
  bm_status rc;
#define BM_KIND2(TT, SS)                                                                         \
  switch (a.kind) {                                                                              \
    case BM_NORM_LAYERNORM: rc = norm_bwd_dispatch<TT, BM_NORM_LAYERNORM, SS>(a, x, stats, dh, dres, dx, h_out, partial, st); break; \
    case BM_NORM_RMSNORM: rc = norm_bwd_dispatch<TT, BM_NORM_RMSNORM, SS>(a, x, stats, dh, dres, dx, h_out, partial, st); break;     \
    default: rc = norm_bwd_dispatch<TT, BM_NORM_ADALN, SS>(a, x, stats, dh, dres, dx, h_out, partial, st); break; \
  }
#define BM_KIND(TT) if (sums) { BM_KIND2(TT, true) } else { BM_KIND2(TT, false) }
  if (a.dtype == BM_DTYPE_BF16) { BM_KIND(bf16_t) } else { BM_KIND(float) }
#undef BM_KIND
#undef BM_KIND2
  BM_RETURN_IF(rc);
  const int nb = norm_bwd_blocks(a.T, a.d);
  if (a.kind == BM_NORM_ADALN) {
    SegArgs p{};
    p.a = dh; p.b = x; p.stats = stats; p.cu = cu_dev; p.out = dmod; p.ld_out = a.ld_mod;
    p.off0 = a.shift_off; p.off1 = a.scale_off; p.rows = a.T; p.N = a.d;
    char* seg_ws = (char*)scratch + align_up((size_t)nb * 4 * a.d * sizeof(float), 256);
    BM_RETURN_IF(seg_launch<1>(a.dtype, p, S, seg_ws, st));
  }
  ReduceTargets t;
  int np = 0;
  float* outs[4] = {nullptr, nullptr, nullptr, nullptr};
  if (a.kind != BM_NORM_ADALN) outs[np++] = dgamma;
  if (a.kind == BM_NORM_LAYERNORM) outs[np++] = dbeta;
  if (sums) { outs[np++] = dsum_res; outs[np++] = dsum_out; }
  if (np == 0) return BM_OK;
  for (int i = 0; i < 4; ++i) { t.partial[i] = partial + (size_t)(i < np ? i : 0) * a.d; t.out[i] = outs[i < np ? i : 0]; }
  hipLaunchKernelGGL(partial_reduce_multi_kernel, dim3(cdiv(a.d, 64), np), dim3(64 * PR_GROUPS), 0, st,
                     t, nb, np * a.d, a.d);
  BM_CHECK_LAUNCH("norm_bwd_reduce");
  return BM_OK;
}

// ------------------------------------------------------------------ RoPE
// One thread owns VEC rotation pairs (i .. i+VEC-1, and the same + dh/2) of one
// token and walks the heads, so each angle is evaluated once per token.
template <typename T>
__global__ void rope_kernel(T* __restrict__ qkv, int ld, int T_rows, int n_heads, int dh,
                            float log2_base, const int32_t* __restrict__ cu,
                            const int32_t* __restrict__ tok_seq, float sign) {
  constexpr int VEC = Elt<T>::VEC;
  const int half = dh >> 1;
  const int chunks = half / VEC;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)T_rows * chunks) return;
  const int t = (int)(gid / chunks);
  const int i0 = (int)(gid % chunks) * VEC;
  const int pos = t - cu[tok_seq[t]];
  float cs[VEC], sn[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    // angle = pos * base^(-2i/dh), evaluated and range-reduced in fp64
    double inv_freq = exp2(-2.0 * (double)(i0 + e) / (double)dh * (double)log2_base);
    double ang = (double)pos * inv_freq;
    const double two_pi = 6.283185307179586476925286766559;
    ang -= two_pi * rint(ang / two_pi);
    float s, c;
    sincosf((float)ang, &s, &c);
    cs[e] = c; sn[e] = sign * s;
  }
  T* row = qkv + (size_t)t * ld;
  for (int hd = 0; hd < n_heads; ++hd) {
    T* p = row + hd * dh + i0;
    float a[VEC], b[VEC], ra[VEC], rb[VEC];
    load16(p, a); load16(p + half, b);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      ra[e] = a[e] * cs[e] - b[e] * sn[e];
      rb[e] = b[e] * cs[e] + a[e] * sn[e];
    }
    store16(p, ra); store16(p + half, rb);
  }
}

bm_status rope_inplace(int dtype, void* qkv, int ld, int T, int n_heads, int dh, float base,
                       const int32_t* cu_dev, const int32_t* tok_seq, float sign, hipStream_t st) {
  if (T == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if ((dh / 2) % vec != 0) { set_error("rope: head_dim %d unsupported", dh); return BM_ERR_UNSUPPORTED; }
  long n = (long)T * ((dh / 2) / vec);
  float log2_base = log2f(base);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (bf16_t*)qkv, ld,
                       T, n_heads, dh, log2_base, cu_dev, tok_seq, sign);
  else
    hipLaunchKernelGGL(rope_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (float*)qkv, ld, T,
                       n_heads, dh, log2_base, cu_dev, tok_seq, sign);
  BM_CHECK_LAUNCH("rope");
  return BM_OK;
}

// ------------------------------------------------------------------ activations
// Phi(z) = (1 + erf(z / sqrt 2)) / 2 and phi(z) = exp(-z^2/2) / sqrt(2 pi) from ONE
// exponential: erfc(x) = (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0
// (Abramowitz & Stegun 7.1.26, absolute error below 1.5e-7, i.e. fp32 rounding level),
// and exp(-x^2) with x = |z| / sqrt 2 is the exponential of the density.
__device__ inline void normal_cdf_pdf(float z, float* cdf, float* pdf) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  const float e = __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);
  float poly = fmaf(t, 1.061405429f, -1.453152027f);
  poly = fmaf(t, poly, 1.421413741f);
  poly = fmaf(t, poly, -0.284496736f);
  poly = fmaf(t, poly, 0.254829592f);
  const float half_erfc = 0.5f * t * poly * e;
  *cdf = z >= 0.f ? 1.0f - half_erfc : half_erfc;
  *pdf = e * 0.39894228040143268f;
}
__device__ inline float gelu_f(float z) {
  float cdf, pdf;
  normal_cdf_pdf(z, &cdf, &pdf);
  return z * cdf;
}
__device__ inline float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }

template <typename T, int ACT>
__global__ void act_fwd_kernel(const T* __restrict__ up, T* __restrict__ a, int rows, int F) {
  constexpr int VEC = Elt<T>::VEC;
  const int per_row = F / VEC;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)rows * per_row) return;
  const long t = gid / per_row;
  const int c = (int)(gid % per_row) * VEC;
  float out[VEC];
  if (ACT == BM_ACT_GELU) {
    float z[VEC];
    load16(up + t * F + c, z);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = gelu_f(z[e]);
  } else {
    float g[VEC], u[VEC];
    load16(up + t * 2 * F + c, g); load16(up + t * 2 * F + F + c, u);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = g[e] * sigmoid_f(g[e]) * u[e];
  }
  store16(a + t * F + c, out);
}

// Backward of the activation over a (column span, row chunk) grid: writes the
// gradient of the pre-activation, optionally the activation output again (the
// weight-gradient GEMM of the down projection reads it) and, with COLSUM, one
// partial column sum of the written gradient per row chunk (bias gradient).
template <typename T, int ACT, bool COLSUM>
__global__ __launch_bounds__(256) void act_bwd_kernel(const T* __restrict__ up, const T* __restrict__ da,
                                                      T* __restrict__ dup, T* __restrict__ a_out,
                                                      float* __restrict__ partial, int rows, int F) {
  constexpr int VEC = Elt<T>::VEC;
  __shared__ float sm[COLSUM ? 4 : 1][WAVE * VEC];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = (blockIdx.x * WAVE + lane) * VEC;
  const int chunks = gridDim.y;
  const int per = (rows + chunks - 1) / chunks;
  const int r0 = blockIdx.y * per;
  const int r1 = min(rows, r0 + per);
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  if (c < F) {
    // two rows per trip: all loads of both rows are issued before any arithmetic
    for (long t = r0 + wave; t < r1; t += 8) {
      constexpr int NIN = ACT == BM_ACT_GELU ? 1 : 2;
      float d[2][VEC], in[2][NIN][VEC];
      const bool two = t + 4 < r1;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !two) break;
        const long tt = t + 4 * h;
        load16(da + tt * F + c, d[h]);
        if (ACT == BM_ACT_GELU) {
          load16(up + tt * F + c, in[h][0]);
        } else {
          load16(up + tt * 2 * F + c, in[h][0]);
          load16(up + tt * 2 * F + F + c, in[h][NIN - 1]);
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !two) break;
        const long tt = t + 4 * h;
        if (ACT == BM_ACT_GELU) {
          float out[VEC], act[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const float z = in[h][0][e];
            float cdf, pdf;
            normal_cdf_pdf(z, &cdf, &pdf);
            out[e] = d[h][e] * (cdf + z * pdf);
            act[e] = z * cdf;
            if (COLSUM) acc[e] += Elt<T>::to_f(Elt<T>::from_f(out[e]));
          }
          store16(dup + tt * F + c, out);
          if (a_out) store16(a_out + tt * F + c, act);
        } else {
          float dg[VEC], du[VEC], act[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const float g = in[h][0][e], u = in[h][NIN - 1][e];
            float sg = sigmoid_f(g);
            dg[e] = d[h][e] * u * sg * (1.0f + g * (1.0f - sg));
            du[e] = d[h][e] * g * sg;
            act[e] = g * sg * u;
          }
          store16(dup + tt * 2 * F + c, dg); store16(dup + tt * 2 * F + F + c, du);
          if (a_out) store16(a_out + tt * F + c, act);
        }
      }
    }
  }
  if (COLSUM) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) sm[wave][lane * VEC + e] = acc[e];
    __syncthreads();
    if (wave == 0 && c < F) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        int i = lane * VEC + e;
        partial[(size_t)blockIdx.y * F + c + e] = sm[0][i] + sm[1][i] + sm[2][i] + sm[3][i];
      }
    }
  }
}

bm_status act_forward(int dtype, int act, const void* up, void* a, int T, int F, hipStream_t st) {
  if (T == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (F % vec) { set_error("activation: mlp_hidden %d not a multiple of %d", F, vec); return BM_ERR_UNSUPPORTED; }
  long n = (long)T * (F / vec);
  dim3 grid(cdiv(n, 256)), block(256);
#define BM_L(TT, AA) hipLaunchKernelGGL((act_fwd_kernel<TT, AA>), grid, block, 0, st, (const TT*)up, (TT*)a, T, F)
  if (dtype == BM_DTYPE_BF16) { if (act == BM_ACT_GELU) BM_L(bf16_t, BM_ACT_GELU); else BM_L(bf16_t, BM_ACT_SWIGLU); }
  else { if (act == BM_ACT_GELU) BM_L(float, BM_ACT_GELU); else BM_L(float, BM_ACT_SWIGLU); }
#undef BM_L
  BM_CHECK_LAUNCH("act_fwd");
  return BM_OK;
}

static void colsum_plan(int T, int N, int vec, int* spans, int* chunks);

// a_out (nullable): the activation output, written again.  bias_grad (nullable,
// GELU only): fp32 [F] that receives += the column sums of dup; scratch then
// needs colsum_scratch_bytes(T, F).
bm_status act_backward(int dtype, int act, const void* up, const void* da, void* dup, void* a_out,
                       float* bias_grad, void* scratch, int T, int F, hipStream_t st) {
  if (T == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (F % vec) { set_error("activation: mlp_hidden %d not a multiple of %d", F, vec); return BM_ERR_UNSUPPORTED; }
  if (bias_grad && act != BM_ACT_GELU) { set_error("activation: bias gradient with a gated MLP"); return BM_ERR_UNSUPPORTED; }
  int spans, chunks;
  colsum_plan(T, F, vec, &spans, &chunks);
  dim3 grid(spans, chunks), block(256);
  float* partial = (float*)scratch;
#define BM_L(TT, AA, CS) hipLaunchKernelGGL((act_bwd_kernel<TT, AA, CS>), grid, block, 0, st, (const TT*)up, (const TT*)da, (TT*)dup, (TT*)a_out, partial, T, F)
  if (dtype == BM_DTYPE_BF16) {
    if (act != BM_ACT_GELU) BM_L(bf16_t, BM_ACT_SWIGLU, false);
    else if (bias_grad) BM_L(bf16_t, BM_ACT_GELU, true);
    else BM_L(bf16_t, BM_ACT_GELU, false);
  } else {
    if (act != BM_ACT_GELU) BM_L(float, BM_ACT_SWIGLU, false);
    else if (bias_grad) BM_L(float, BM_ACT_GELU, true);
    else BM_L(float, BM_ACT_GELU, false);
  }
#undef BM_L
  if (bias_grad)
    hipLaunchKernelGGL(partial_reduce_kernel, dim3(cdiv(F, 64)), dim3(64 * PR_GROUPS), 0, st, partial, chunks, F,
                       F, bias_grad);
  BM_CHECK_LAUNCH("act_bwd");
  return BM_OK;
}

// ------------------------------------------------------------------ column sums (bias grads)
// stage 1: grid (column spans, row chunks); a wavefront reads 64*VEC contiguous
// columns of one row per step.  stage 2: fixed-order sum of the chunk partials.
static void colsum_plan(int T, int N, int vec, int* spans, int* chunks) {
  *spans = cdiv(N, WAVE * vec);
  int r = cdiv(1024, *spans);
  int rmax = cdiv(T, 4);
  if (r > rmax) r = rmax;
  if (r > 256) r = 256;
  if (r < 1) r = 1;
  *chunks = r;
}

size_t colsum_scratch_bytes(int T, int N) {
  // chunks * N <= 1024 * 64 * VEC + N for any width up to N, and chunks <= 256
  (void)T;
  size_t bound = (size_t)1024 * 512 + N;
  size_t cap = (size_t)256 * N;
  return (bound < cap ? bound : cap) * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1_kernel(const T* __restrict__ a, int lda, int rows,
                                                            int N, float* __restrict__ partial) {
  constexpr int VEC = Elt<T>::VEC;
  __shared__ float sm[4][WAVE * VEC];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = (blockIdx.x * WAVE + lane) * VEC;
  const int chunks = gridDim.y;
  const int per = (rows + chunks - 1) / chunks;
  const int r0 = blockIdx.y * per;
  const int r1 = min(rows, r0 + per);
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  if (col < N) {
    for (int r = r0 + wave; r < r1; r += 4) {
      float v[VEC];
      load16(a + (size_t)r * lda + col, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) sm[wave][lane * VEC + e] = acc[e];
  __syncthreads();
  if (wave == 0 && col < N) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      int i = lane * VEC + e;
      partial[(size_t)blockIdx.y * N + col + e] = sm[0][i] + sm[1][i] + sm[2][i] + sm[3][i];
    }
  }
}

bm_status colsum_accumulate(int dtype, const void* a, int lda, int T, int N, float* out,
                            void* scratch, hipStream_t st) {
  if (T == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  if (N % vec || lda % vec) { set_error("colsum: width %d/%d not a multiple of %d", N, lda, vec); return BM_ERR_UNSUPPORTED; }
  int spans, chunks;
  colsum_plan(T, N, vec, &spans, &chunks);
  float* partial = (float*)scratch;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(colsum_stage1_kernel<bf16_t>, dim3(spans, chunks), dim3(256), 0, st,
                       (const bf16_t*)a, lda, T, N, partial);
  else
    hipLaunchKernelGGL(colsum_stage1_kernel<float>, dim3(spans, chunks), dim3(256), 0, st,
                       (const float*)a, lda, T, N, partial);
  hipLaunchKernelGGL(partial_reduce_kernel, dim3(cdiv(N, 64)), dim3(64 * PR_GROUPS), 0, st, partial, chunks, N,
                     N, out);
  BM_CHECK_LAUNCH("colsum");
  return BM_OK;
}

// ------------------------------------------------------------------ small elementwise helpers
template <typename T>
__global__ void gate_mul_kernel(const T* __restrict__ a, const float* __restrict__ gate, int ld_gate,
                                const int32_t* __restrict__ tok_seq, const T* __restrict__ residual,
                                T* __restrict__ out, int rows, int N) {
  constexpr int VEC = Elt<T>::VEC;
  const int per_row = N / VEC;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)rows * per_row) return;
  const long t = gid / per_row;
  const int c = (int)(gid % per_row) * VEC;
  const float* g = gate + (size_t)tok_seq[t] * ld_gate + c;
  float v[VEC];
  load16(a + t * N + c, v);
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] *= g[e];
  if (residual) {
    float r[VEC];
    load16(residual + t * N + c, r);
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] += r[e];
  }
  store16(out + t * N + c, v);
}

bm_status gate_mul(int dtype, const void* a, const float* gate, int ld_gate, const int32_t* tok_seq,
                   const void* residual, void* out, int T, int N, hipStream_t st) {
  if (T == 0) return BM_OK;
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  long n = (long)T * (N / vec);
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(gate_mul_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st,
                       (const bf16_t*)a, gate, ld_gate, tok_seq, (const bf16_t*)residual, (bf16_t*)out, T, N);
  else
    hipLaunchKernelGGL(gate_mul_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st,
                       (const float*)a, gate, ld_gate, tok_seq, (const float*)residual, (float*)out, T, N);
  BM_CHECK_LAUNCH("gate_mul");
  return BM_OK;
}

template <typename T>
__global__ void silu_fwd_kernel(const T* __restrict__ in, T* __restrict__ out, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float z = Elt<T>::to_f(in[i]);
  out[i] = Elt<T>::from_f(z * sigmoid_f(z));
}

template <typename T>
__global__ void silu_bwd_f32_kernel(const T* __restrict__ in, const float* __restrict__ g,
                                    T* __restrict__ out, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float z = Elt<T>::to_f(in[i]);
  float s = sigmoid_f(z);
  out[i] = Elt<T>::from_f(g[i] * s * (1.0f + z * (1.0f - s)));
}

template <typename T>
__global__ void cast_from_f32_kernel(const float* __restrict__ in, T* __restrict__ out, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = Elt<T>::from_f(in[i]);
}

// out[n, s] = in[s, n] for s < rows, 0 for rows <= s < ld_out
template <typename T>
__global__ void cast_transpose_from_f32_kernel(const float* __restrict__ in, T* __restrict__ out, int rows,
                                               int cols, int ld_out) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)cols * ld_out) return;
  const int n = (int)(i / ld_out), s = (int)(i % ld_out);
  out[i] = Elt<T>::from_f(s < rows ? in[(size_t)s * cols + n] : 0.f);
}

bm_status cast_transpose_from_f32(int dtype, const float* in, void* out, int rows, int cols, int ld_out,
                                  hipStream_t st) {
  const long n = (long)cols * ld_out;
  if (n == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(cast_transpose_from_f32_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, in,
                       (bf16_t*)out, rows, cols, ld_out);
  else
    hipLaunchKernelGGL(cast_transpose_from_f32_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, in,
                       (float*)out, rows, cols, ld_out);
  BM_CHECK_LAUNCH("cast_transpose");
  return BM_OK;
}

bm_status silu_forward(int dtype, const void* in, void* out, long n, hipStream_t st) {
  if (n == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(silu_fwd_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const bf16_t*)in, (bf16_t*)out, n);
  else
    hipLaunchKernelGGL(silu_fwd_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const float*)in, (float*)out, n);
  BM_CHECK_LAUNCH("silu_fwd");
  return BM_OK;
}

bm_status silu_backward_f32(int dtype, const void* in, const float* g, void* out, long n, hipStream_t st) {
  if (n == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(silu_bwd_f32_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const bf16_t*)in, g, (bf16_t*)out, n);
  else
    hipLaunchKernelGGL(silu_bwd_f32_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, (const float*)in, g, (float*)out, n);
  BM_CHECK_LAUNCH("silu_bwd");
  return BM_OK;
}

bm_status cast_from_f32(int dtype, const float* in, void* out, long n, hipStream_t st) {
  if (n == 0) return BM_OK;
  if (dtype == BM_DTYPE_BF16)
    hipLaunchKernelGGL(cast_from_f32_kernel<bf16_t>, dim3(cdiv(n, 256)), dim3(256), 0, st, in, (bf16_t*)out, n);
  else
    hipLaunchKernelGGL(cast_from_f32_kernel<float>, dim3(cdiv(n, 256)), dim3(256), 0, st, in, (float*)out, n);
  BM_CHECK_LAUNCH("cast");
  return BM_OK;
}

}  // namespace bm
