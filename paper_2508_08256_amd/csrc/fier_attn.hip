// Exact attention over a selected subset of K/V rows (Alg. 1 step 4), and over the whole cache when no
// index list is given (the decode attention of Sec. 3.1).
//
// Split-K: workgroup (split, unit) owns `rows_per_wg` consecutive entries of the unit's selection and
// produces one partial (m, l, o[128]) per query head; a second kernel merges the partials with the
// usual running-max rescale.  Inside a workgroup a row of 16 lanes owns one K/V row at a time: lane n of
// the row loads channels 8n..8n+7 as one 16-byte request, so a wavefront fetches 4 whole 256-byte rows
// per load instruction and 4 such loads (16 rows) of K and of V are in flight per iteration.  The
// q.k products use the packed 16-bit dot instructions with binary32 accumulation, are reduced over the
// 16 lanes with DPP rotates, and softmax / PV run in binary32 with exp2.
#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

constexpr int kAttnUnroll = 4;                  // rows per 16-lane row per iteration
constexpr int kRowsPerIter = 4 * 4 * kAttnUnroll;  // 4 waves x 4 lane rows x unroll

template <int DT, int NREP>
__global__ __launch_bounds__(256) void attn_split_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                         const uint4* __restrict__ q, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ seq_lens, int extra,
                                                         int max_budget, int rows_per_wg, int n_splits,
                                                         float scale_log2e, float* __restrict__ po,
                                                         float* __restrict__ pm, float* __restrict__ pl,
                                                         int n_kv_heads, int max_ctx) {
  __shared__ float sh_o[16][16][8 + 2];  // [wave*4 + lane row][channel chunk][o[8], m, l]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int rs = lane >> 4, cn = lane & 15;
  const int unit = blockIdx.y, split = blockIdx.x;
  const int b = unit / n_kv_heads;
  int n;
  if (idx) {
    n = count[unit];
    n = n > max_budget ? max_budget : n;
  } else {
    n = seq_lens[b] + extra;
    n = n > max_ctx ? max_ctx : n;
  }
  const int start = split * rows_per_wg;
  if (start >= n) return;
  const int end = n < start + rows_per_wg ? n : start + rows_per_wg;
  const int32_t* __restrict__ sel = idx ? idx + (size_t)unit * max_budget : nullptr;
  const uint4* __restrict__ Ku = K + (size_t)unit * max_ctx * (kD / 8);
  const uint4* __restrict__ Vu = V + (size_t)unit * max_ctx * (kD / 8);

  uint4 qr[NREP];
#pragma unroll
  for (int r = 0; r < NREP; ++r) qr[r] = q[((size_t)unit * NREP + r) * (kD / 8) + cn];

  float m_run[NREP], l_run[NREP], o[NREP][8];
#pragma unroll
  for (int r = 0; r < NREP; ++r) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[r][c] = 0.f;
  }

  for (int i0 = start + wave * (4 * kAttnUnroll); i0 < end; i0 += kRowsPerIter) {
    uint4 kk[kAttnUnroll], vv[kAttnUnroll];
    bool valid[kAttnUnroll];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int j = i0 + u * 4 + rs;
      valid[u] = j < end;
      int t = valid[u] ? (sel ? sel[j] : j) : 0;
      t = (t < 0 || t >= max_ctx) ? 0 : t;
      kk[u] = Ku[(size_t)t * (kD / 8) + cn];
      vv[u] = Vu[(size_t)t * (kD / 8) + cn];
    }
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
      float logit[kAttnUnroll];
      float mx = m_run[r];
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        float d = dot2<DT>(kk[u].x, qr[r].x, 0.f);
        d = dot2<DT>(kk[u].y, qr[r].y, d);
        d = dot2<DT>(kk[u].z, qr[r].z, d);
        d = dot2<DT>(kk[u].w, qr[r].w, d);
        d = row_allsum(d);
        logit[u] = valid[u] ? d * scale_log2e : -INFINITY;
        mx = fmaxf(mx, logit[u]);
      }
      const float mref = mx == -INFINITY ? 0.f : mx;
      const float alpha = __builtin_amdgcn_exp2f(m_run[r] - mref);
      float p[kAttnUnroll], psum = 0.f;
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        p[u] = __builtin_amdgcn_exp2f(logit[u] - mref);
        psum += p[u];
      }
      m_run[r] = mx;
      l_run[r] = l_run[r] * alpha + psum;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[r][c] *= alpha;
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        const uint32_t vw[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          o[r][2 * c] += p[u] * lo16f<DT>(vw[c]);
          o[r][2 * c + 1] += p[u] * hi16f<DT>(vw[c]);
        }
      }
    }
  }

  // combine the 16 (wave, lane row) states of the workgroup per query head and channel
#pragma unroll
  for (int r = 0; r < NREP; ++r) {
    if (r > 0) __syncthreads();
    float* dst = sh_o[wave * 4 + rs][cn];
#pragma unroll
    for (int c = 0; c < 8; ++c) dst[c] = o[r][c];
    dst[8] = m_run[r];
    dst[9] = l_run[r];
    __syncthreads();
    if (tid < kD) {
      const int chunk = tid >> 3, e = tid & 7;
      float M = -INFINITY;
#pragma unroll
      for (int s = 0; s < 16; ++s) M = fmaxf(M, sh_o[s][chunk][8]);
      float acc = 0.f, lsum = 0.f;
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        const float ms = sh_o[s][chunk][8];
        const float w = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - M);
        acc += w * sh_o[s][chunk][e];
        lsum += w * sh_o[s][chunk][9];
      }
      const size_t slot = ((size_t)unit * NREP + r) * n_splits + split;
      po[slot * kD + tid] = acc;
      if (tid == 0) {
        pm[slot] = M;
        pl[slot] = lsum;
      }
    }
  }
}

// grid (units * n_rep), block 128: thread c merges channel c of one query head over the splits in use.
__global__ __launch_bounds__(128) void attn_merge_kernel(const float* __restrict__ po, const float* __restrict__ pm,
                                                         const float* __restrict__ pl,
                                                         const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ seq_lens, int extra,
                                                         int max_budget, int rows_per_wg, int n_splits, int n_rep,
                                                         float* __restrict__ out, int n_kv_heads, int max_ctx) {
  const int head = blockIdx.x;  // unit * n_rep + r
  const int unit = head / n_rep;
  const int b = unit / n_kv_heads;
  int n;
  if (count) {
    n = count[unit];
    n = n > max_budget ? max_budget : n;
  } else {
    n = seq_lens[b] + extra;
    n = n > max_ctx ? max_ctx : n;
  }
  const int c = threadIdx.x;
  if (n <= 0) {
    out[(size_t)head * kD + c] = 0.f;
    return;
  }
  const int used = (n + rows_per_wg - 1) / rows_per_wg;
  const size_t base = (size_t)head * n_splits;
  float M = -INFINITY;
  for (int s = 0; s < used; ++s) M = fmaxf(M, pm[base + s]);
  float acc = 0.f, lsum = 0.f;
  for (int s = 0; s < used; ++s) {
    const float w = __builtin_amdgcn_exp2f(pm[base + s] - M);
    acc += w * po[(base + s) * kD + c];
    lsum += w * pl[base + s];
  }
  out[(size_t)head * kD + c] = acc / lsum;
}

template <int DT>
static hipError_t launch_attn_dt(int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                                 const int32_t* count, const int32_t* seq_lens, int extra, int max_budget,
                                 int rows_per_wg, int n_splits, float sm_scale, float* po, float* pm, float* pl,
                                 int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  dim3 grid(n_splits, units);
  const float sl2 = sm_scale * 1.4426950408889634f;
#define FIER_ATTN_CASE(R)                                                                                          \
  case R:                                                                                                          \
    attn_split_kernel<DT, R><<<grid, 256, 0, st>>>((const uint4*)K, (const uint4*)V, (const uint4*)q, idx, count,  \
                                                   seq_lens, extra, max_budget, rows_per_wg, n_splits, sl2, po, pm, \
                                                   pl, n_kv_heads, max_ctx);                                       \
    break;
  switch (n_rep) {
    FIER_ATTN_CASE(1)
    FIER_ATTN_CASE(2)
    FIER_ATTN_CASE(3)
    FIER_ATTN_CASE(4)
    FIER_ATTN_CASE(5)
    FIER_ATTN_CASE(6)
    FIER_ATTN_CASE(7)
    FIER_ATTN_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_ATTN_CASE
  return hipGetLastError();
}

hipError_t launch_attn(int dtype, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                       const int32_t* count, const int32_t* seq_lens, int extra, int max_budget, int rows_per_wg,
                       int n_splits, float sm_scale, float* po, float* pm, float* pl, float* out, int units,
                       int n_kv_heads, int max_ctx, hipStream_t st) {
  hipError_t e;
  if (dtype == DT_F16)
    e = launch_attn_dt<DT_F16>(n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                               sm_scale, po, pm, pl, units, n_kv_heads, max_ctx, st);
  else
    e = launch_attn_dt<DT_BF16>(n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                                sm_scale, po, pm, pl, units, n_kv_heads, max_ctx, st);
  if (e != hipSuccess) return e;
  attn_merge_kernel<<<units * n_rep, 128, 0, st>>>(po, pm, pl, idx ? count : nullptr, seq_lens, extra, max_budget,
                                                   rows_per_wg, n_splits, n_rep, out, n_kv_heads, max_ctx);
  return hipGetLastError();
}

}  // namespace fier
