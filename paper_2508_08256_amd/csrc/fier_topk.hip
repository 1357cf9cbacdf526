// Top-B token selection per unit (Alg. 1 step 3): the B largest scores, ties to the lower index,
// indices emitted in ascending order.
//
// One 1024-thread workgroup per unit; everything except the scores themselves lives in LDS.
//   1. min / max of the scores.
//   2. value-space histogram: 2048 equal-width bins between min and max.  (A radix pass over the raw
//      float bits would put most scores of one magnitude into a handful of bins and serialise the
//      LDS atomics; equal-width bins spread a bell-shaped score distribution.)
//   3. the bin holding the B-th largest score is found with a suffix scan; its members are the only
//      candidates for the threshold, their order-preserving integer keys are gathered into LDS.
//   4. exact radix select (4 x 8 bits) among the candidates gives the threshold key T and the number
//      r of tokens equal to T that still fit.
//   5. one ordered pass writes every index with key > T, and the first r with key == T.
// All decisions are integer comparisons of keys, so the result is exact and deterministic.
#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

constexpr int kTkThreads = 1024;
constexpr int kTkWaves = kTkThreads / 64;
constexpr int kTkBins = 2048;
constexpr int kTkCandMax = 8192;

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane) { return wave_incl_scan_u32(v, lane); }

// Exclusive scan of one value per thread over the workgroup (thread order); also returns the total.
// `tmp` is kTkWaves words of LDS; contains two barriers.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* tmp, uint32_t& total) {
  return block_excl_scan_u32<kTkWaves>(v, tmp, total);
}

template <bool IsMax>
__device__ __forceinline__ float block_minmax(float v, float* tmp) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    float o = __shfl_xor(v, d, 64);
    v = IsMax ? fmaxf(v, o) : fminf(v, o);
  }
  __syncthreads();
  if (lane == 0) tmp[wave] = v;
  __syncthreads();
  float r = tmp[0];
#pragma unroll
  for (int w = 1; w < kTkWaves; ++w) r = IsMax ? fmaxf(r, tmp[w]) : fminf(r, tmp[w]);
  return r;
}

// Find in hist[0..nb) (counts per bin, ascending value order) the bin b such that
// (count in bins > b) < want <= (count in bins >= b).  Returns b and the count above it.
// nb <= 2 * kTkThreads.  Contains barriers; result valid in every thread.
__device__ __forceinline__ void find_bin_from_top(const uint32_t* hist, int nb, uint32_t want, uint32_t* tmp,
                                                  int* res, int& bin, uint32_t& above) {
  const int t = threadIdx.x;
  // thread t owns the two bins nb-1-2t and nb-2-2t (descending order)
  const int b0 = nb - 1 - 2 * t, b1 = nb - 2 - 2 * t;
  const uint32_t c0 = b0 >= 0 ? hist[b0] : 0, c1 = b1 >= 0 ? hist[b1] : 0;
  uint32_t total;
  const uint32_t before = block_excl_scan(c0 + c1, tmp, total);
  if (before < want && want <= before + c0) {
    res[0] = b0;
    res[1] = (int)before;
  } else if (before + c0 < want && want <= before + c0 + c1) {
    res[0] = b1;
    res[1] = (int)(before + c0);
  }
  __syncthreads();
  bin = res[0];
  above = (uint32_t)res[1];
}

// bin of the equal-width histogram; monotone non-decreasing in v
__device__ __forceinline__ int value_bin(float v, float lo, float scale) {
  return (int)fminf(fmaxf((v - lo) * scale, 0.0f), (float)(kTkBins - 1));  // clamped before the conversion
}

// Visit the unit's scores as 16-byte chunks: chunk c of thread tid covers tokens (c * 1024 + tid) * 4 .. + 3.
// NV > 0: the chunks were loaded into registers once; NV == 0: they are streamed from memory on every visit.
// Entries at or past n hold unspecified data: the visitor masks them with the token index.
template <int NV, class F>
__device__ __forceinline__ void for_chunks(const float4 (&regs)[NV > 0 ? NV : 1], const float* __restrict__ s, int n,
                                           int max_ctx, F&& f) {
  const int tid = threadIdx.x;
  if constexpr (NV > 0) {
#pragma unroll
    for (int c = 0; c < NV; ++c)
      if (c * 4 * kTkThreads < n) f(c, regs[c], (c * kTkThreads + tid) * 4);
  } else {
    const int nch = (n + 4 * kTkThreads - 1) / (4 * kTkThreads);
#pragma unroll 4
    for (int c = 0; c < nch; ++c) {
      const int i = (c * kTkThreads + tid) * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < max_ctx) v = *reinterpret_cast<const float4*>(s + i);
      f(c, v, i);
    }
  }
}

// NV > 0: register-resident variant for max_ctx <= NV * 4096; NV == 0: streaming variant for any length.
template <int NV>
__global__ __launch_bounds__(kTkThreads) void topk_kernel(const float* __restrict__ scores,
                                                          const int32_t* __restrict__ seq_lens, int extra,
                                                          const int32_t* __restrict__ budgets, int max_budget,
                                                          int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                          int n_kv_heads, int max_ctx) {
  constexpr int NVR = NV > 0 ? NV : 1;
  __shared__ uint32_t hist[kTkBins];
  __shared__ uint32_t cand[kTkCandMax];
  __shared__ uint32_t scan_tmp[kTkWaves + 1];
  __shared__ float red_tmp[kTkWaves];
  __shared__ int res[2];
  __shared__ uint32_t n_cand_sh;
  __shared__ uint32_t thr_sh[2];
  __shared__ uint32_t wtot[NVR * kTkWaves];
  __shared__ uint32_t offg[NVR * kTkWaves], offe[NVR * kTkWaves];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x;
  const int b = unit / n_kv_heads;
  int n = seq_lens[b] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  int B = budgets[b];
  B = B > max_budget ? max_budget : B;
  B = B > n ? n : B;
  const float* __restrict__ s = scores + (size_t)unit * max_ctx;
  int32_t* __restrict__ out = idx + (size_t)unit * max_budget;
  if (B <= 0) {
    if (tid == 0) count[unit] = 0;
    return;
  }
  if (tid == 0) count[unit] = B;
  if (B >= n) {  // the whole context is selected
    for (int i = tid; i < n; i += kTkThreads) out[i] = i;
    return;
  }

  float4 regs[NVR];
  if constexpr (NV > 0) {
#pragma unroll
    for (int c = 0; c < NV; ++c) {
      const int i = (c * kTkThreads + tid) * 4;
      regs[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (c * 4 * kTkThreads < n && i < max_ctx) regs[c] = *reinterpret_cast<const float4*>(s + i);
    }
  }

  // ---- 1. range of the scores ----------------------------------------------------------------
  float lo = INFINITY, hi = -INFINITY;
  for_chunks<NV>(regs, s, n, max_ctx, [&](int, const float4 v, int i) {
    const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j < n) {
        lo = fminf(lo, vv[j]);
        hi = fmaxf(hi, vv[j]);
      }
  });
  lo = block_minmax<false>(lo, red_tmp);
  hi = block_minmax<true>(hi, red_tmp);

  uint32_t T;      // threshold key
  uint32_t r_eq;   // how many tokens with key == T are selected (the lowest indices)
  if (!(hi > lo)) {
    T = score_key(lo);
    r_eq = (uint32_t)B;
  } else {
    // ---- 2. equal-width histogram ------------------------------------------------------------
    const float scale = (float)kTkBins / (hi - lo);
    for (int i = tid; i < kTkBins; i += kTkThreads) hist[i] = 0;
    if (tid == 0) n_cand_sh = 0;
    __syncthreads();
    for_chunks<NV>(regs, s, n, max_ctx, [&](int, const float4 v, int i) {
      const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i + j < n) atomicAdd(&hist[value_bin(vv[j], lo, scale)], 1u);
    });
    __syncthreads();
    // ---- 3. threshold bin and its candidates -------------------------------------------------
    int tbin;
    uint32_t above;
    find_bin_from_top(hist, kTkBins, (uint32_t)B, scan_tmp, res, tbin, above);
    uint32_t r = (uint32_t)B - above;      // rank of the threshold inside the bin, 1-based from the top
    const uint32_t n_cand = hist[tbin];
    const bool in_lds = n_cand <= (uint32_t)kTkCandMax;
    __syncthreads();
    if (in_lds) {
      for_chunks<NV>(regs, s, n, max_ctx, [&](int, const float4 v, int i) {
        const float vv[4] = {v.x, v.y, v.z, v.w};
        bool is_c[4];
        uint32_t cnt = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          is_c[j] = i + j < n && value_bin(vv[j], lo, scale) == tbin;
          cnt += is_c[j];
        }
        if (cnt) {
          uint32_t pos = atomicAdd(&n_cand_sh, cnt);
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (is_c[j]) cand[pos++] = score_key(vv[j]);
        }
      });
      __syncthreads();
    }
    if (n_cand <= 512u) {
      // ---- 4a. few candidates: rank each one against all others ------------------------------
      if ((uint32_t)tid < n_cand) {
        const uint32_t key = cand[tid];
        uint32_t gt = 0, ge = 0;
        for (uint32_t j = 0; j < n_cand; ++j) {
          const uint32_t o = cand[j];
          gt += o > key;
          ge += o >= key;
        }
        if (gt < r && r <= ge) {  // every thread holding the threshold value writes the same pair
          thr_sh[0] = key;
          thr_sh[1] = r - gt;
        }
      }
      __syncthreads();
      T = thr_sh[0];
      r_eq = thr_sh[1];
    } else {
      // ---- 4b. exact radix select of the r-th largest candidate key --------------------------
      uint32_t prefix = 0, mask = 0;
#pragma unroll 1
      for (int pass = 3; pass >= 0; --pass) {
        const int shift = 8 * pass;
        for (int i = tid; i < 256; i += kTkThreads) hist[i] = 0;
        __syncthreads();
        if (in_lds) {
          for (uint32_t i = tid; i < n_cand; i += kTkThreads) {
            const uint32_t key = cand[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
          }
        } else {  // more candidates than LDS holds (heavily clustered scores): stream them from memory
          for (int i = tid; i < n; i += kTkThreads) {
            const float v = s[i];
            const uint32_t key = score_key(v);
            if (value_bin(v, lo, scale) == tbin && (key & mask) == prefix)
              atomicAdd(&hist[(key >> shift) & 255u], 1u);
          }
        }
        __syncthreads();
        int dbin;
        uint32_t dabove;
        find_bin_from_top(hist, 256, r, scan_tmp, res, dbin, dabove);
        r -= dabove;
        prefix |= (uint32_t)dbin << shift;
        mask |= 0xffu << shift;
        __syncthreads();
      }
      T = prefix;
      r_eq = r;
    }
  }

  // ---- 5. ordered emission ---------------------------------------------------------------------
  // token order = (chunk, thread, element).  A token is selected iff key > T, or key == T and fewer than
  // r_eq equal keys precede it; its output slot is the number of selected tokens before it.
  if constexpr (NV > 0) {
    // all chunks at once: per-wave scans of every chunk's counts, one scan over the (chunk, wave) totals
    uint32_t cnt[NV], incl[NV];
#pragma unroll
    for (int c = 0; c < NV; ++c) {
      const int i = (c * kTkThreads + tid) * 4;
      const float vv[4] = {regs[c].x, regs[c].y, regs[c].z, regs[c].w};
      uint32_t cg = 0, ce = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = score_key(vv[j]);
        const bool ok = i + j < n;
        cg += ok && key > T;
        ce += ok && key == T;
      }
      cnt[c] = cg | (ce << 16);
      incl[c] = wave_incl_scan(cnt[c], lane);
    }
    if (lane == 63) {
#pragma unroll
      for (int c = 0; c < NV; ++c) wtot[c * kTkWaves + wave] = incl[c];
    }
    __syncthreads();
    if (wave == 0) {
      constexpr int ENT = NV * kTkWaves;
      constexpr int PER = (ENT + 63) / 64;
      uint32_t g[PER], e[PER], sg = 0, se = 0;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const int ent = lane * PER + k;
        const uint32_t w = ent < ENT ? wtot[ent] : 0;
        g[k] = w & 0xffffu;
        e[k] = w >> 16;
        sg += g[k];
        se += e[k];
      }
      uint32_t pg = wave_incl_scan(sg, lane) - sg, pe = wave_incl_scan(se, lane) - se;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const int ent = lane * PER + k;
        if (ent < ENT) {
          offg[ent] = pg;
          offe[ent] = pe;
        }
        pg += g[k];
        pe += e[k];
      }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NV; ++c) {
      if (c * 4 * kTkThreads >= n) continue;
      const int i = (c * kTkThreads + tid) * 4;
      const float vv[4] = {regs[c].x, regs[c].y, regs[c].z, regs[c].w};
      const uint32_t ex = incl[c] - cnt[c];
      uint32_t g_before = offg[c * kTkWaves + wave] + (ex & 0xffffu);
      uint32_t e_before = offe[c * kTkWaves + wave] + (ex >> 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = score_key(vv[j]);
        const bool ok = i + j < n;
        const bool gt = ok && key > T, eq = ok && key == T;
        if (gt || (eq && e_before < r_eq)) out[g_before + (e_before < r_eq ? e_before : r_eq)] = i + j;
        g_before += gt;
        e_before += eq;
      }
    }
  } else {
    uint32_t run_gt = 0, run_eq = 0;  // counts over all earlier tokens (uniform across the workgroup)
    for (int i0 = 0; i0 < n; i0 += 4 * kTkThreads) {
      const int i = i0 + 4 * tid;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < max_ctx) v = *reinterpret_cast<const float4*>(s + i);
      const float vv[4] = {v.x, v.y, v.z, v.w};
      uint32_t gt[4], eq[4], cg = 0, ce = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t key = score_key(vv[j]);
        const bool ok = i + j < n;
        gt[j] = ok && key > T;
        eq[j] = ok && key == T;
        cg += gt[j];
        ce += eq[j];
      }
      uint32_t total;
      const uint32_t ex = block_excl_scan(cg | (ce << 16), scan_tmp, total);
      uint32_t g_before = run_gt + (ex & 0xffffu);
      uint32_t e_before = run_eq + (ex >> 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (gt[j] || (eq[j] && e_before < r_eq)) out[g_before + (e_before < r_eq ? e_before : r_eq)] = i + j;
        g_before += gt[j];
        e_before += eq[j];
      }
      run_gt += total & 0xffffu;
      run_eq += total >> 16;
    }
  }
}

hipError_t launch_topk(const float* scores, const int32_t* seq_lens, int extra, const int32_t* budgets,
                       int max_budget, int32_t* idx, int32_t* count, int units, int n_kv_heads, int max_ctx,
                       hipStream_t st) {
#define FIER_TOPK(NV)                                                                                           \
  topk_kernel<NV><<<units, kTkThreads, 0, st>>>(scores, seq_lens, extra, budgets, max_budget, idx, count, \
                                                n_kv_heads, max_ctx)
  const int chunks = (max_ctx + 4 * kTkThreads - 1) / (4 * kTkThreads);
  if (chunks <= 2)
    FIER_TOPK(2);
  else if (chunks <= 4)
    FIER_TOPK(4);
  else if (chunks <= 9)
    FIER_TOPK(9);
  else
    FIER_TOPK(0);
#undef FIER_TOPK
  return hipGetLastError();
}

// ---- the same selection by many workgroups per unit (long contexts) ----------------------------------------------------
// Four small kernels on the fused step's machinery: (1) largest |score| per unit = the histogram range R,
// (2) 512-bin histogram of the scores over [-R, R], (3) the fused step's threshold kernel (exact threshold among the
// candidates of the threshold bin, offsets of the 1024-token ranges in the ascending index list), (4) emission of the
// indices range by range.  All decisions are the same integer comparisons as above: the result is identical.

// grid (units, ceil(max_ctx / 4096)), block 1024: thread t looks at tokens 4t..4t+3 of the workgroup's stretch.
// (Units vary fastest in the dispatch order of all four kernels: a unit's workgroups share an XCD and its L2.)
__global__ __launch_bounds__(1024) void topk_absmax_kernel(const float* __restrict__ scores,
                                                           const int32_t* __restrict__ seq_lens, int extra,
                                                           UnitCtl* __restrict__ ctl, int n_kv_heads, int max_ctx) {
  __shared__ float tmp[kTkWaves];
  const int unit = blockIdx.x, chunk = blockIdx.y;
  int n = seq_lens[unit / n_kv_heads] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  const int i = chunk * kClassifyTokens + 4 * (int)threadIdx.x;
  if (chunk * kClassifyTokens >= n) return;
  float m = 0.f;
  if (i < n) {
    const float4 v = *reinterpret_cast<const float4*>(scores + (size_t)unit * max_ctx + i);
    m = fabsf(v.x);
    if (i + 1 < n) m = fmaxf(m, fabsf(v.y));
    if (i + 2 < n) m = fmaxf(m, fabsf(v.z));
    if (i + 3 < n) m = fmaxf(m, fabsf(v.w));
  }
  m = block_minmax<true>(m, tmp);
  // non-negative floats order like their bit patterns; the slot is zero between calls
  if (threadIdx.x == 0 && m > 0.f) atomicMax(&ctl[unit].topk_max, __float_as_uint(m));
}

// Same grid.  Bins its stretch into an LDS histogram and adds it to the unit's; the unit's first workgroup also
// publishes the range the scores are binned with, where the threshold kernel expects it.
__global__ __launch_bounds__(1024) void topk_hist_kernel(const float* __restrict__ scores,
                                                         const int32_t* __restrict__ seq_lens, int extra,
                                                         UnitCtl* __restrict__ ctl, uint32_t* __restrict__ ghist,
                                                         int n_kv_heads, int max_ctx) {
  __shared__ uint32_t lhist[kSelBins];
  const int unit = blockIdx.x, chunk = blockIdx.y, tid = threadIdx.x;
  int n = seq_lens[unit / n_kv_heads] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  float R = __uint_as_float(ctl[unit].topk_max);
  R = R > 0.f ? R : 1.0f;  // all scores zero: any range will do
  const float scale = (float)kSelBins / (R + R);
  if (chunk == 0 && tid == 0) {
    ctl[unit].R = R;
    ctl[unit].scale = scale;
  }
  if (chunk * kClassifyTokens >= n) return;
  if (tid < kSelBins) lhist[tid] = 0;
  __syncthreads();
  const int i = chunk * kClassifyTokens + 4 * tid;
  if (i < n) {
    const float4 v = *reinterpret_cast<const float4*>(scores + (size_t)unit * max_ctx + i);
    const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j < n) atomicAdd(&lhist[sel_bin(vv[j], R, scale, kSelBins)], 1u);
  }
  __syncthreads();
  if (tid < kSelBins && lhist[tid]) atomicAdd(&ghist[(size_t)unit * kSelBins + tid], lhist[tid]);
}

// grid (units, n_ranges), block 256: the selected tokens of one 1024-token range, in token order, at the offset the
// threshold kernel computed for the range.
__global__ __launch_bounds__(256) void topk_emit_kernel(const float* __restrict__ scores,
                                                        const int32_t* __restrict__ seq_lens, int extra,
                                                        UnitCtl* __restrict__ ctl,
                                                        const uint32_t* __restrict__ range_off, int max_budget,
                                                        int32_t* __restrict__ idx, int n_ranges, int n_kv_heads,
                                                        int max_ctx) {
  __shared__ uint32_t scan_tmp[4];
  const int unit = blockIdx.x, r = blockIdx.y, tid = threadIdx.x;
  int n = seq_lens[unit / n_kv_heads] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  UnitCtl* __restrict__ c = &ctl[unit];
  if (r == 0 && tid == 0) c->topk_max = 0;  // every reader of it has finished (earlier kernels)
  const int i = r * kRangeTokens + 4 * tid;
  if (r * kRangeTokens >= n) return;
  const int tbin = c->tbin;
  const float R = c->R, scale = c->scale;
  const uint32_t T = c->T;
  const int32_t idxT = c->idxT;
  const uint32_t off = range_off[(size_t)unit * n_ranges + r];
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n) v = *reinterpret_cast<const float4*>(scores + (size_t)unit * max_ctx + i);
  const float vv[4] = {v.x, v.y, v.z, v.w};
  uint32_t selm = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int bin = sel_bin(vv[j], R, scale, kSelBins);
    const uint32_t key = score_key(vv[j]);
    const bool sel = i + j < n && (bin > tbin || (bin == tbin && (key > T || (key == T && i + j <= idxT))));
    selm |= sel ? 1u << j : 0u;
  }
  uint32_t total;
  uint32_t pos = off + block_excl_scan_u32<4>((uint32_t)__builtin_popcount(selm), scan_tmp, total);
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (selm >> j & 1u) {
      if (pos < (uint32_t)max_budget) idx[(size_t)unit * max_budget + pos] = i + j;
      ++pos;
    }
}

hipError_t launch_topk_ws(const StepBuffers& sb_in, const float* scores, const int32_t* seq_lens, int extra,
                          const int32_t* budgets, int max_budget, int32_t* idx, int32_t* count, int units,
                          int n_kv_heads, int max_ctx, hipStream_t st) {
  if (max_ctx <= 9 * 4 * kTkThreads)  // the scores of a unit fit one workgroup's registers: one kernel is faster
    return launch_topk(scores, seq_lens, extra, budgets, max_budget, idx, count, units, n_kv_heads, max_ctx, st);
  StepBuffers sb = sb_in;
  sb.scores = const_cast<float*>(scores);  // the threshold kernel only reads them
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  dim3 grid4k(units, (max_ctx + kClassifyTokens - 1) / kClassifyTokens);
  topk_absmax_kernel<<<grid4k, 1024, 0, st>>>(scores, seq_lens, extra, sb.ctl, n_kv_heads, max_ctx);
  topk_hist_kernel<<<grid4k, 1024, 0, st>>>(scores, seq_lens, extra, sb.ctl, sb.hist, n_kv_heads, max_ctx);
  hipError_t e = launch_threshold(sb, seq_lens, extra, budgets, max_budget, count, units, n_kv_heads, max_ctx, st);
  if (e != hipSuccess) return e;
  topk_emit_kernel<<<dim3(units, n_ranges), 256, 0, st>>>(scores, seq_lens, extra, sb.ctl, sb.range_cnt, max_budget,
                                                          idx, n_ranges, n_kv_heads, max_ctx);
  return hipGetLastError();
}

}  // namespace fier
