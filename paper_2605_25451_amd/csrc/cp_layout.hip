// Host-side planning of the encoder -> LLM context-parallel layout conversion, the encoder unit
// size under different context-parallel degrees, and the C-ABI face of the row moves that apply
// a plan on device memory.
#include "common.h"
#include "../../include/bigmac_cp_attention.h"

#include <algorithm>
#include <vector>

namespace bm {

namespace {

// first position of chunk c of a sequence of length L cut into C ranges
inline long chunk_begin(long L, int C, int c) { return (long)c * L / C; }

// chunk that holds position p
inline int chunk_of(long L, int C, long p) {
  int c = (int)(p * C / L);
  if (c > C - 1) c = C - 1;
  while (p < chunk_begin(L, C, c)) --c;
  while (p >= chunk_begin(L, C, c + 1)) ++c;
  return c;
}

// base[s*C + c]: local row on rank c where its chunk of sequence s starts
void chunk_bases(const std::vector<long>& lens, int C, std::vector<long>& base) {
  std::vector<long> fill(C, 0);
  base.assign(lens.size() * C, 0);
  for (size_t s = 0; s < lens.size(); ++s)
    for (int c = 0; c < C; ++c) {
      base[s * C + c] = fill[c];
      fill[c] += chunk_begin(lens[s], C, c + 1) - chunk_begin(lens[s], C, c);
    }
}

}  // namespace

}  // namespace bm

using namespace bm;

extern "C" bm_status bm_cp_conversion_plan(int32_t enc_cp, int32_t llm_cp, int32_t n_images,
                                           const int32_t* image_lens, const int32_t* image_rows,
                                           int32_t n_docs, const int32_t* cu_docs, int32_t* counts,
                                           int32_t* src_rows, int32_t* dst_rows) {
  BM_ARG_CHECK(enc_cp >= 1 && llm_cp >= 1, "cp plan: degrees %d / %d", enc_cp, llm_cp);
  BM_ARG_CHECK(n_images >= 0 && n_docs >= 1, "cp plan: %d images, %d documents", n_images, n_docs);
  BM_ARG_CHECK(cu_docs && counts && (n_images == 0 || image_lens), "cp plan: NULL argument");
  BM_ARG_CHECK(cu_docs[0] == 0, "cp plan: document offsets must start at 0");
  std::vector<long> ilen(n_images), dlen(n_docs);
  long N = 0;
  for (int i = 0; i < n_images; ++i) {
    BM_ARG_CHECK(image_lens[i] >= 0, "cp plan: image %d has length %d", i, image_lens[i]);
    ilen[i] = image_lens[i]; N += ilen[i];
  }
  for (int d = 0; d < n_docs; ++d) {
    BM_ARG_CHECK(cu_docs[d + 1] >= cu_docs[d], "cp plan: document %d has a negative length", d);
    dlen[d] = cu_docs[d + 1] - cu_docs[d];
  }
  const long T = cu_docs[n_docs];
  BM_ARG_CHECK(N == 0 || (image_rows && src_rows && dst_rows), "cp plan: NULL row arrays");
  std::vector<char> seen(T, 0);
  for (long k = 0; k < N; ++k) {
    BM_ARG_CHECK(image_rows[k] >= 0 && image_rows[k] < T, "cp plan: token %ld goes to row %d outside the pack of %ld rows", k, image_rows[k], T);
    BM_ARG_CHECK(!seen[image_rows[k]], "cp plan: row %d is filled twice", image_rows[k]);
    seen[image_rows[k]] = 1;
  }
  std::vector<long> ebase, lbase;
  chunk_bases(ilen, enc_cp, ebase);
  chunk_bases(dlen, llm_cp, lbase);
  // per token: pair index and the two local rows
  std::vector<int32_t> pair(N), src(N), dst(N);
  std::vector<long> cnt((size_t)enc_cp * llm_cp, 0);
  long k = 0;
  for (int i = 0; i < n_images; ++i)
    for (long p = 0; p < ilen[i]; ++p, ++k) {
      const int e = chunk_of(ilen[i], enc_cp, p);
      const long r = image_rows[k];
      const int d = (int)(std::upper_bound(cu_docs, cu_docs + n_docs + 1, (int32_t)r) - cu_docs) - 1;
      const long q = r - cu_docs[d];
      const int l = chunk_of(dlen[d], llm_cp, q);
      pair[k] = e * llm_cp + l;
      src[k] = (int32_t)(ebase[(size_t)i * enc_cp + e] + p - chunk_begin(ilen[i], enc_cp, e));
      dst[k] = (int32_t)(lbase[(size_t)d * llm_cp + l] + q - chunk_begin(dlen[d], llm_cp, l));
      ++cnt[pair[k]];
    }
  // stable grouping by pair: inside a pair tokens stay in (image, position) order, which is
  // ascending source-row order on the sending rank
  std::vector<long> at(cnt.size(), 0);
  long run = 0;
  for (size_t g = 0; g < cnt.size(); ++g) { at[g] = run; run += cnt[g]; counts[g] = (int32_t)cnt[g]; }
  for (long t = 0; t < N; ++t) {
    const long o = at[pair[t]]++;
    src_rows[o] = src[t];
    dst_rows[o] = dst[t];
  }
  return BM_OK;
}

extern "C" bm_status bm_cp_encoder_unit_size(int32_t pp_size, int32_t llm_cp, int32_t enc_cp, int32_t* unit_size) {
  BM_ARG_CHECK(pp_size >= 1 && llm_cp >= 1 && enc_cp >= 1 && unit_size, "cp unit size: bad argument");
  const long n = (long)pp_size * llm_cp;
  BM_ARG_CHECK(n % enc_cp == 0, "cp unit size: pp_size * llm_cp = %ld is not a multiple of enc_cp = %d", n, enc_cp);
  *unit_size = (int32_t)(n / enc_cp);
  return BM_OK;
}

static bm_status check_rows(int32_t dtype, const void* src, const int32_t* rows, void* dst, int32_t n, int32_t width) {
  BM_ARG_CHECK(dtype == BM_DTYPE_BF16 || dtype == BM_DTYPE_FP32, "row move: dtype %d", dtype);
  const int vec = dtype == BM_DTYPE_BF16 ? 8 : 4;
  BM_ARG_CHECK(n >= 0 && width > 0 && width % vec == 0, "row move: n = %d, width = %d", n, width);
  BM_ARG_CHECK(n == 0 || (src && rows && dst), "row move: NULL argument");
  BM_ARG_CHECK(n == 0 || (((uintptr_t)src | (uintptr_t)dst) & 15) == 0, "row move: misaligned tensor");
  return BM_OK;
}

extern "C" bm_status bm_row_gather(int32_t dtype, const void* src, const int32_t* rows_dev, void* dst, int32_t n,
                                   int32_t width, void* hip_stream) {
  BM_RETURN_IF(check_rows(dtype, src, rows_dev, dst, n, width));
  return row_gather(dtype, src, rows_dev, dst, n, width, (hipStream_t)hip_stream);
}

extern "C" bm_status bm_row_scatter(int32_t dtype, const void* src, const int32_t* rows_dev, void* dst, int32_t n,
                                    int32_t width, void* hip_stream) {
  BM_RETURN_IF(check_rows(dtype, src, rows_dev, dst, n, width));
  return row_scatter(dtype, src, rows_dev, dst, n, width, (hipStream_t)hip_stream);
}
