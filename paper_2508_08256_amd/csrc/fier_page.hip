// Page-level importance: the page-retrieval baseline the paper compares with (Sec. 3.2, Eq. 1-3) and its
// "averaged quantized score per page" ablation (Sec. 4.4), as a second workload for the top-k and gather kernels.
//
// A page = P consecutive tokens of one unit (P = 8, 16 or 32).  Its metadata are the channel-wise minimum and
// maximum key vectors over the tokens present: page_meta [units][max_ctx / P][128] uint32 = min | max << 16 in the
// K dtype (input values, hence exact) -- 512 bytes per page, the load ratio 2 / P of the paper (1/8 at P = 16).
//   page score, mode 0 (Eq. 3 as printed): max over the channels of max(q_i kmax_i, q_i kmin_i);
//   page score, mode 1: the same summed over the channels, an upper bound of q . k for every key of the page;
//   with several query heads per kv head the per-head page scores are added.
#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

// grid (ceil(n_pages / 4), units), block 256: one wavefront per page, lane = channel pair.
template <int DT>
__global__ __launch_bounds__(256) void page_minmax_kernel(const uint32_t* __restrict__ K,
                                                          const int32_t* __restrict__ seq_lens,
                                                          uint32_t* __restrict__ page_meta, int n_kv_heads,
                                                          int max_ctx, int P, KvLayout lay) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int unit = blockIdx.y;
  const int n_pages = max_ctx / P;
  const int p = blockIdx.x * 4 + wave;
  if (p >= n_pages) return;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int t0 = p * P;
  uint2 res = make_uint2(0, 0);
  if (t0 < L) {
    const int nt = L - t0 < P ? L - t0 : P;
    const uint32_t* src = K + lay.rows_of(unit).row(t0) * (kD / 2) + lane;  // a page lies inside one block
    uint32_t w = src[0];
    uint32_t mn0 = w & 0xffffu, mx0 = mn0, mn1 = w >> 16, mx1 = mn1;
    for (int t = 1; t < nt; ++t) {
      w = src[(size_t)t * (kD / 2)];
      const uint32_t a = w & 0xffffu, b = w >> 16;
      if (w2f<DT>(a) < w2f<DT>(mn0)) mn0 = a;
      if (w2f<DT>(a) > w2f<DT>(mx0)) mx0 = a;
      if (w2f<DT>(b) < w2f<DT>(mn1)) mn1 = b;
      if (w2f<DT>(b) > w2f<DT>(mx1)) mx1 = b;
    }
    res = make_uint2(mn0 | (mx0 << 16), mn1 | (mx1 << 16));
  }
  reinterpret_cast<uint2*>(page_meta + ((size_t)unit * n_pages + p) * kD)[lane] = res;
}

// grid (units), block 64: the row just written at position L = seq_len joins its page.
template <int DT>
__global__ __launch_bounds__(64) void page_append_kernel(const uint32_t* __restrict__ k_new,
                                                         const int32_t* __restrict__ seq_lens,
                                                         uint32_t* __restrict__ page_meta, int n_kv_heads,
                                                         int max_ctx, int P) {
  const int lane = threadIdx.x, unit = blockIdx.x;
  const int L = seq_lens[unit / n_kv_heads];
  if (L < 0 || L >= max_ctx) return;
  const int n_pages = max_ctx / P;
  const uint32_t w = k_new[(size_t)unit * (kD / 2) + lane];
  const uint32_t a = w & 0xffffu, b = w >> 16;
  uint2* dst = reinterpret_cast<uint2*>(page_meta + ((size_t)unit * n_pages + L / P) * kD) + lane;
  uint32_t mn0 = a, mx0 = a, mn1 = b, mx1 = b;
  if (L % P != 0) {  // the page already holds tokens
    const uint2 old = *dst;
    mn0 = old.x & 0xffffu, mx0 = old.x >> 16, mn1 = old.y & 0xffffu, mx1 = old.y >> 16;
    if (w2f<DT>(a) < w2f<DT>(mn0)) mn0 = a;
    if (w2f<DT>(a) > w2f<DT>(mx0)) mx0 = a;
    if (w2f<DT>(b) < w2f<DT>(mn1)) mn1 = b;
    if (w2f<DT>(b) > w2f<DT>(mx1)) mx1 = b;
  }
  *dst = make_uint2(mn0 | (mx0 << 16), mn1 | (mx1 << 16));
}

// grid (ceil(n_pages / 64), units), block 256: a 16-lane row scores one page at a time (lane cn the channels
// 8cn..8cn+7: two 16-byte loads of the page's 512 bytes), 4 pages per row.  The products of two 16-bit floats are
// exact in binary32, so mode 0 is exact; mode 1 adds 128 of them per head in binary32.
template <int DT, int NREP>
__global__ __launch_bounds__(256) void page_score_kernel(const uint4* __restrict__ page_meta,
                                                         const uint4* __restrict__ q,
                                                         const int32_t* __restrict__ seq_lens, int extra, int mode,
                                                         float* __restrict__ out, int n_kv_heads, int max_ctx,
                                                         int P) {
  const int tid = threadIdx.x;
  const int cn = tid & 15, rowid = tid >> 4;  // 16 rows of 16 lanes
  const int unit = blockIdx.y;
  const int n_pages = max_ctx / P;
  int L = seq_lens[unit / n_kv_heads] + extra;
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  float qf[NREP][8];
#pragma unroll
  for (int h = 0; h < NREP; ++h) {
    const uint4 qq = q[((size_t)unit * NREP + h) * (kD / 8) + cn];
    const uint32_t qw[4] = {qq.x, qq.y, qq.z, qq.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      qf[h][2 * c] = lo16f<DT>(qw[c]);
      qf[h][2 * c + 1] = hi16f<DT>(qw[c]);
    }
  }
#pragma unroll 1
  for (int it = 0; it < 4; ++it) {
    const int p = blockIdx.x * 64 + it * 16 + rowid;
    if (p >= n_pages) break;
    float total = -INFINITY;
    if (p * P < L) {
      const uint4* src = page_meta + ((size_t)unit * n_pages + p) * (kD / 4) + 2 * cn;  // 8 channels = 8 words
      const uint4 m0 = src[0], m1 = src[1];
      const uint32_t mw[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
      total = 0.f;
#pragma unroll
      for (int h = 0; h < NREP; ++h) {
        float acc = mode == 0 ? -INFINITY : 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const float a_min = qf[h][c] * lo16f<DT>(mw[c]);
          const float a_max = qf[h][c] * hi16f<DT>(mw[c]);
          const float m = fmaxf(a_max, a_min);
          acc = mode == 0 ? fmaxf(acc, m) : acc + m;
        }
        if (mode == 0) {
          acc = fmaxf(acc, row_ror<8>(acc));
          acc = fmaxf(acc, row_ror<4>(acc));
          acc = fmaxf(acc, row_ror<2>(acc));
          acc = fmaxf(acc, row_ror<1>(acc));
        } else {
          acc = row_allsum(acc);
        }
        total += acc;
      }
    }
    if (cn == 0) out[(size_t)unit * n_pages + p] = total;
  }
}

// grid (ceil(n_pages / 256), units), block 256: thread = page, the average of its tokens' scores (P <= 32).
__global__ __launch_bounds__(256) void page_mean_kernel(const float* __restrict__ scores,
                                                        const int32_t* __restrict__ seq_lens, int extra,
                                                        float* __restrict__ out, int n_kv_heads, int max_ctx, int P) {
  const int unit = blockIdx.y;
  const int n_pages = max_ctx / P;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= n_pages) return;
  int L = seq_lens[unit / n_kv_heads] + extra;
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int t0 = p * P;
  float r = -INFINITY;
  if (t0 < L) {
    const int nt = L - t0 < P ? L - t0 : P;
    const float* s = scores + (size_t)unit * max_ctx + t0;
    float acc = 0.f;
    for (int t = 0; t < nt; ++t) acc += s[t];
    r = acc / (float)nt;
  }
  out[(size_t)unit * n_pages + p] = r;
}

// grid (units), block 256: all tokens of the selected pages (ascending page list), clipped to the length.  Only
// the last page of a sequence can be partial and it can only be last in the list, so entry k starts at k * P.
__global__ __launch_bounds__(256) void expand_pages_kernel(const int32_t* __restrict__ page_idx,
                                                           const int32_t* __restrict__ page_count, int max_pages,
                                                           const int32_t* __restrict__ seq_lens, int extra, int P,
                                                           int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                           int max_budget, int n_kv_heads, int max_ctx) {
  const int unit = blockIdx.x;
  int L = seq_lens[unit / n_kv_heads] + extra;
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  int n = page_count[unit];
  n = n < 0 ? 0 : (n > max_pages ? max_pages : n);
  const int32_t* pl = page_idx + (size_t)unit * max_pages;
  for (int e = threadIdx.x; e < n * P; e += 256) {
    const int k = e / P, j = e - k * P;
    const int t = pl[k] * P + j;
    if (t >= 0 && t < L && e < max_budget) idx[(size_t)unit * max_budget + e] = t;
  }
  if (threadIdx.x == 0) {
    int c = 0;
    if (n > 0) {
      const int last = pl[n - 1];
      int in_last = L - last * P;
      in_last = in_last > P ? P : (in_last < 0 ? 0 : in_last);
      c = (n - 1) * P + in_last;
    }
    count[unit] = c > max_budget ? max_budget : c;
  }
}

hipError_t launch_page_minmax(int dtype, KvLayout lay, const void* K, const int32_t* seq_lens, uint32_t* page_meta, int units,
                              int n_kv_heads, int max_ctx, int P, hipStream_t st) {
  dim3 grid((max_ctx / P + 3) / 4, units);
  if (dtype == DT_F16)
    page_minmax_kernel<DT_F16><<<grid, 256, 0, st>>>((const uint32_t*)K, seq_lens, page_meta, n_kv_heads, max_ctx, P,
                                                     lay);
  else
    page_minmax_kernel<DT_BF16><<<grid, 256, 0, st>>>((const uint32_t*)K, seq_lens, page_meta, n_kv_heads, max_ctx, P,
                                                     lay);
  return hipGetLastError();
}

hipError_t launch_page_append(int dtype, const void* k_new, const int32_t* seq_lens, uint32_t* page_meta, int units,
                              int n_kv_heads, int max_ctx, int P, hipStream_t st) {
  if (dtype == DT_F16)
    page_append_kernel<DT_F16><<<units, 64, 0, st>>>((const uint32_t*)k_new, seq_lens, page_meta, n_kv_heads, max_ctx,
                                                     P);
  else
    page_append_kernel<DT_BF16><<<units, 64, 0, st>>>((const uint32_t*)k_new, seq_lens, page_meta, n_kv_heads,
                                                      max_ctx, P);
  return hipGetLastError();
}

template <int DT>
static hipError_t launch_page_score_dt(int n_rep, const uint32_t* page_meta, const void* q, const int32_t* seq_lens,
                                       int extra, int mode, float* out, int units, int n_kv_heads, int max_ctx,
                                       int P, hipStream_t st) {
  dim3 grid((max_ctx / P + 63) / 64, units);
#define FIER_PS_CASE(R)                                                                                           \
  case R:                                                                                                         \
    page_score_kernel<DT, R><<<grid, 256, 0, st>>>((const uint4*)page_meta, (const uint4*)q, seq_lens, extra, mode, \
                                                   out, n_kv_heads, max_ctx, P);                                  \
    break;
  switch (n_rep) {
    FIER_PS_CASE(1)
    FIER_PS_CASE(2)
    FIER_PS_CASE(3)
    FIER_PS_CASE(4)
    FIER_PS_CASE(5)
    FIER_PS_CASE(6)
    FIER_PS_CASE(7)
    FIER_PS_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_PS_CASE
  return hipGetLastError();
}

hipError_t launch_page_score(int dtype, int n_rep, const uint32_t* page_meta, const void* q, const int32_t* seq_lens,
                             int extra, int mode, float* out, int units, int n_kv_heads, int max_ctx, int P,
                             hipStream_t st) {
  if (dtype == DT_F16)
    return launch_page_score_dt<DT_F16>(n_rep, page_meta, q, seq_lens, extra, mode, out, units, n_kv_heads, max_ctx,
                                        P, st);
  return launch_page_score_dt<DT_BF16>(n_rep, page_meta, q, seq_lens, extra, mode, out, units, n_kv_heads, max_ctx, P,
                                       st);
}

hipError_t launch_page_mean(const float* scores, const int32_t* seq_lens, int extra, float* out, int units,
                            int n_kv_heads, int max_ctx, int P, hipStream_t st) {
  dim3 grid((max_ctx / P + 255) / 256, units);
  page_mean_kernel<<<grid, 256, 0, st>>>(scores, seq_lens, extra, out, n_kv_heads, max_ctx, P);
  return hipGetLastError();
}

hipError_t launch_expand_pages(const int32_t* page_idx, const int32_t* page_count, int max_pages,
                               const int32_t* seq_lens, int extra, int P, int32_t* idx, int32_t* count,
                               int max_budget, int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  expand_pages_kernel<<<units, 256, 0, st>>>(page_idx, page_count, max_pages, seq_lens, extra, P, idx, count,
                                             max_budget, n_kv_heads, max_ctx);
  return hipGetLastError();
}

}  // namespace fier
