// Second kernel of the fused decode step: exact top-B threshold per unit (Alg. 1 step 3).
//
// The score kernel has left, per unit, the 512-bin histogram of its scores.  Every workgroup here first finds,
// from that histogram, the bin `tbin` that contains the B-th largest score and the number of scores in bins
// above it (the same few hundred integer additions in every workgroup of the unit: cheaper than a serial step at
// the end of the score kernel plus the wait for it), then re-reads 4096 scores of its unit and
//   * counts, per 1024-token range, the tokens in bins above tbin (they are selected for certain);
//   * writes the tokens that fall into tbin itself -- the only candidates for the threshold, about 1 % of
//     the tokens for bell-shaped scores -- as (key, index) pairs into its own candidate segment.
// The unit's last workgroup gathers the segments into LDS, histograms the candidates once more inside the
// threshold bin (1024 sub-bins), ranks the handful of members of the decisive sub-bin pairwise (larger key
// first, equal keys by lower index), which fixes the threshold key T and the last selected index idxT among
// equal keys, and turns the per-range counts into the exclusive offsets at which the next kernel writes the
// ascending index list.  If the candidates do not fit (scores clustered far more tightly than the a-priori
// range resolves), the last workgroup falls back to a radix selection streamed over the unit's scores.
#include "fier_dev.h"
#include "fier_kernels.h"
#include "fier_select_dev.h"

namespace fier {

constexpr int kThrThreads = 1024;
constexpr int kThrWaves = kThrThreads / 64;
constexpr int kMaxRanges = (1 << 20) / kRangeTokens;  // max_ctx <= 2^20
constexpr int kMaxChunks = (1 << 20) / kClassifyTokens;
constexpr int kSpecCand = 64;                          // candidates per segment fetched before its count is known

// grid (units, ceil(max_ctx / (4096 NV))), block 1024: a workgroup classifies NV stretches of 4096 tokens (thread t
// the tokens 4t..4t+3 of each).  The launcher picks NV so that all workgroups are resident at once if possible.
// Units vary fastest in the dispatch order: workgroups go round-robin to the 8 XCDs, so with a multiple of 8 units
// all workgroups of a unit run on one XCD and its histogram, candidate segments and counters stay in that XCD's L2
// (measured against chunks-fastest: 9.9 -> 8.4 us at config 2, 21.1 -> 16.5 us for the ragged 128-unit batch).
template <int NV>
__global__ __launch_bounds__(kThrThreads) void threshold_kernel(const float* __restrict__ scores,
                                                                const int32_t* __restrict__ seq_lens, int extra,
                                                                UnitCtl* __restrict__ ctl,
                                                                uint32_t* __restrict__ ghist,
                                                                const int32_t* __restrict__ budgets, int max_budget,
                                                                uint32_t* __restrict__ range_cnt,
                                                                unsigned long long* __restrict__ cand,
                                                                uint32_t* __restrict__ seg_cnt,
                                                                int32_t* __restrict__ count_out, int n_ranges,
                                                                int n_chunks, int tail_tokens, int n_kv_heads,
                                                                int max_ctx) {
  __shared__ uint32_t wsum[NV + 1][kThrWaves];  // the last row: a folded tail range
  __shared__ uint32_t flag;
  __shared__ int found[2];
  __shared__ uint32_t scan_tmp[kThrWaves];
  __shared__ uint32_t hist[kSubBins];
  __shared__ uint32_t res[2];
  __shared__ uint32_t n_local;
  __shared__ uint32_t n_sub;
  __shared__ unsigned long long lcand[kSelCandMax];
  __shared__ unsigned long long sub_list[kSubCandMax];
  __shared__ uint32_t rsel[kMaxRanges];
  __shared__ uint32_t seg_base[kMaxChunks];  // one segment per classifying workgroup
  __shared__ uint32_t seg_size[kMaxChunks];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x, chunk = blockIdx.y;
  const int b = unit / n_kv_heads;
  int n = seq_lens[b] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  constexpr int kChunkTokens = kClassifyTokens * NV;
  if (chunk * kChunkTokens >= n && chunk != 0) return;
  FIER_PROF(10, unit == 0 && chunk == 1)
  FIER_PROF_WG(2)
  UnitCtl* __restrict__ c = &ctl[unit];
  const float R = c->R, scale = c->scale;
  const float* __restrict__ s = scores + (size_t)unit * max_ctx;
  unsigned long long* __restrict__ ucand = cand + (size_t)unit * n_chunks * kSegCand;
  uint32_t* __restrict__ useg = seg_cnt + (size_t)unit * n_chunks;
  uint32_t* __restrict__ urange = range_cnt + (size_t)unit * n_ranges;
  uint32_t* __restrict__ gh = ghist + (size_t)unit * kSelBins;

  // this workgroup's scores and the unit's histogram leave in the same round trip
  float4 v[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = chunk * kChunkTokens + k * kClassifyTokens + 4 * tid;
    v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n) v[k] = *reinterpret_cast<const float4*>(s + i);  // i + 3 < max_ctx; entries >= n are masked below
  }
  // thread t < 512 owns bin 511 - t: descending score order
  const uint32_t hcnt = tid < kSelBins ? gh[kSelBins - 1 - tid] : 0;
  int B = budgets[b];
  B = B > max_budget ? max_budget : B;
  B = B > n ? n : B;
  B = B < 0 ? 0 : B;
  if (tid == 0) {
    n_local = 0;
    found[0] = B >= n ? -1 : kSelBins;  // everything / nothing selected by bin alone
    found[1] = 0;
  }
  // ---- the bin that holds the B-th largest score ---------------------------------------------------------
  {
    uint32_t total;
    const uint32_t before = block_excl_scan_u32<kThrWaves>(hcnt, scan_tmp, total);  // has barriers
    if (B > 0 && B < n && before < (uint32_t)B && (uint32_t)B <= before + hcnt) {
      found[0] = kSelBins - 1 - tid;
      found[1] = (int)before;
    }
    __syncthreads();
  }
  const int tbin = found[0];
  const uint32_t above = (uint32_t)found[1];

  // ---- classify this workgroup's scores ----------------------------------------------------------------
  FIER_PROF(11, unit == 0 && chunk == 1)
  uint32_t cmask = 0;  // candidate flags: bit 4k + j = token j of stretch k
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = chunk * kChunkTokens + k * kClassifyTokens + 4 * tid;
    const float vv[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
    uint32_t n_gt = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool ok = i + j < n;
      const int bin = sel_bin(vv[j], R, scale, kSelBins);
      n_gt += ok && bin > tbin;
      cmask |= (ok && bin == tbin) ? 1u << (4 * k + j) : 0u;
    }
    // selected-for-certain count of each 1024-token range (4 wavefronts per range)
    const uint32_t g = wave_sum_u32(n_gt);
    if (lane == 0) wsum[k][wave] = g;
  }
  // A last range that would be a workgroup of its own (a capacity of 2^k rows plus the appended one is the common
  // case) -- and with it one more dispatch round for a few tokens per unit -- is classified by the unit's last
  // workgroup instead, one token per thread: tail_tokens (<= 1024) tokens from the end of its chunk.
  const bool takes_tail = tail_tokens > 0 && chunk == n_chunks - 1;
  bool tail_cand = false;
  float tail_x = 0.f;
  if (takes_tail) {
    const int i = (chunk + 1) * kChunkTokens + tid;
    const bool ok = tid < tail_tokens && i < n;
    if (ok) tail_x = s[i];
    const int bin = sel_bin(tail_x, R, scale, kSelBins);
    tail_cand = ok && bin == tbin;
    const uint32_t g = wave_sum_u32(ok && bin > tbin ? 1u : 0u);
    if (lane == 0) wsum[NV][wave] = g;
  }
  // candidates go to this workgroup's own segment; the slot comes from an LDS counter
  if (tail_cand) {
    const uint32_t pos = atomicAdd(&n_local, 1u);
    if (pos < (uint32_t)kSegCand)
      store_coherent(&ucand[(size_t)chunk * kSegCand + pos],
                     ((unsigned long long)score_key(tail_x) << 32) | (uint32_t)((chunk + 1) * kChunkTokens + tid));
  }
  if (cmask) {
    uint32_t pos = atomicAdd(&n_local, (uint32_t)__builtin_popcount(cmask));
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = chunk * kChunkTokens + k * kClassifyTokens + 4 * tid;
      const float vv[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (cmask >> (4 * k + j) & 1u) {
          if (pos < (uint32_t)kSegCand)
            store_coherent(&ucand[(size_t)chunk * kSegCand + pos],
                           ((unsigned long long)score_key(vv[j]) << 32) | (uint32_t)(i + j));
          ++pos;
        }
    }
  }
  __syncthreads();
  if (tid < 4 * NV) {
    const int k = tid >> 2, q4 = tid & 3;
    const int r = chunk * (4 * NV) + tid;
    if (r < n_ranges)
      store_coherent(&urange[r], wsum[k][4 * q4] + wsum[k][4 * q4 + 1] + wsum[k][4 * q4 + 2] + wsum[k][4 * q4 + 3]);
  }
  if (tid == 4 * NV) store_coherent(&useg[chunk], n_local);
  if (takes_tail && tid == 4 * NV + 1) {
    uint32_t g = 0;
#pragma unroll
    for (int w = 0; w < kThrWaves; ++w) g += wsum[NV][w];
    store_coherent(&urange[n_ranges - 1], g);
  }
  int nc = n > 0 ? (n + kChunkTokens - 1) / kChunkTokens : 1;  // workgroups of this unit
  nc = nc > n_chunks ? n_chunks : nc;                            // (a folded tail has none of its own)
  FIER_PROF(12, unit == 0 && chunk == 1)
  FIER_PROF_WG(3)
  if (!last_arriver(&c->arrive[1], (uint32_t)nc, &flag)) return;
  FIER_PROF(13, unit == 0)

  // ---- the unit's last workgroup: exact threshold ------------------------------------------------------
  const int nr = (n + kRangeTokens - 1) / kRangeTokens;  // ranges in use (<= n_ranges)
  const bool need_threshold = tbin >= 0 && tbin < kSelBins && B > 0;
  // segment sizes, and the first candidates of every segment in the same round trip
  uint32_t my_cnt = 0;
  if (tid < nc) my_cnt = load_coherent(&useg[tid]);
  uint32_t my_range = 0;  // ranges tid, tid + 1024, ...: the first one is fetched in the same round trip
  if (tid < nr) my_range = load_coherent(&urange[tid]);
  unsigned long long spec = 0;
  const int sseg = tid / kSpecCand, sk = tid % kSpecCand;
  if (need_threshold && sseg < nc) spec = load_coherent(&ucand[(size_t)sseg * kSegCand + sk]);
  for (int r = tid; r < nr; r += kThrThreads) rsel[r] = 0;
  // exclusive scan of the segment sizes (nc <= 256 for max_ctx <= 2^20; thread t < nc holds segment t)
  bool overflow = false;
  uint32_t total_cand;
  {
    const uint32_t capped = my_cnt > (uint32_t)kSegCand ? (uint32_t)kSegCand : my_cnt;
    const uint32_t before = block_excl_scan_u32<kThrWaves>(capped, scan_tmp, total_cand);
    if (tid < nc) {
      seg_base[tid] = before;
      seg_size[tid] = capped;
    }
    overflow = __syncthreads_or(my_cnt > (uint32_t)kSegCand) || total_cand > (uint32_t)kSelCandMax;
  }
  FIER_PROF(14, unit == 0)
  uint32_t T = 0;
  int32_t idxT = -1;
  if (need_threshold) {
    const uint32_t r_want = (uint32_t)B - above;  // candidates to take, >= 1
    bool done = false;
    if (!overflow) {
      // gather the segments into LDS
      if (sseg < nc) {
        if ((uint32_t)sk < seg_size[sseg]) lcand[seg_base[sseg] + sk] = spec;
      }
      // the rest in one batch of independent loads: flat entry e -> (segment, slot) by binary search of seg_base
      for (uint32_t e = tid; e < total_cand; e += kThrThreads) {
        int lo = 0, hi = nc - 1;
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (seg_base[mid] <= e) lo = mid; else hi = mid - 1;
        }
        const uint32_t k = e - seg_base[lo];
        const bool prefetched = lo < kThrThreads / kSpecCand && k < (uint32_t)kSpecCand;
        if (!prefetched) lcand[e] = load_coherent(&ucand[(size_t)lo * kSegCand + k]);
      }
      __syncthreads();
      done = exact_select_lds<kThrThreads, kSubBins, kSubCandMax>(lcand, total_cand, r_want, tbin, R, scale, hist,
                                                                  sub_list, &n_sub, res, scan_tmp, rsel, T, idxT);
    }
    if (!done) {
      for (int r = tid; r < nr; r += kThrThreads) rsel[r] = 0;
      __syncthreads();
      stream_select<kThrThreads>([&](int k) { return s[k]; }, n, tbin, R, scale, r_want, hist, scan_tmp, res, rsel,
                                 T, idxT);
    }
  }
  __syncthreads();
  FIER_PROF(15, unit == 0)
  // ---- offsets of the ranges in the ascending index list ------------------------------------------------
  uint32_t run = 0;
  for (int r0 = 0; r0 < nr; r0 += kThrThreads) {
    const int r = r0 + tid;
    const uint32_t cnt = r < nr ? (r0 == 0 ? my_range : load_coherent(&urange[r])) + rsel[r] : 0;
    uint32_t total;
    const uint32_t before = run + block_excl_scan_u32<kThrWaves>(cnt, scan_tmp, total);
    if (r < nr) urange[r] = before;
    run += total;
  }
  if (tid < kSelBins) gh[tid] = 0;  // the histogram is zero between calls
  if (tid == 0) {
    c->tbin = tbin;
    c->above = above;
    c->budget = B;
    c->T = T;
    c->idxT = idxT;
    c->arrive[1] = 0;
    if (count_out) count_out[unit] = B;
  }
  FIER_PROF(16, unit == 0)
  FIER_PROF_WG(4)
}

hipError_t launch_threshold(const StepBuffers& sb, const int32_t* seq_lens, int extra, const int32_t* budgets,
                            int max_budget, int32_t* count_out, int units, int n_kv_heads, int max_ctx,
                            hipStream_t st) {
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  // tokens per workgroup: 4096 NV.  One stretch per thread while the grid fits the machine at once (two workgroups
  // of 1024 threads per CU, 256 CUs), two beyond that (measured best at 1000 to 2000 workgroups), four for more
  // than 2048 workgroups of two; the candidate segments are sized for NV = 1 (the most)
  // a last chunk that is a single range goes to the workgroup before it (see the kernel)
  auto folds = [&](int v) { return n_ranges > 1 && (n_ranges - 1) % (4 * v) == 0; };
  auto chunks = [&](int v) {
    return folds(v) ? (n_ranges - 1) / (4 * v) : (max_ctx + kClassifyTokens * v - 1) / (kClassifyTokens * v);
  };
  auto wgs = [&](int v) { return (size_t)units * chunks(v); };
  int nv = 1;
  if (wgs(1) > 512) nv = 2;
  if (wgs(2) > 2048) nv = 4;
  const int n_chunks = chunks(nv);
  const int tail_tokens = folds(nv) ? max_ctx - (n_ranges - 1) * kRangeTokens : 0;
  dim3 grid(units, n_chunks);
#define FIER_THR_CASE(NV)                                                                                            \
  threshold_kernel<NV><<<grid, kThrThreads, 0, st>>>(sb.scores, seq_lens, extra, sb.ctl, sb.hist, budgets,         \
                                                     max_budget, sb.range_cnt, sb.cand, sb.seg_cnt, count_out,      \
                                                     n_ranges, n_chunks, tail_tokens, n_kv_heads, max_ctx)
  if (nv == 1)
    FIER_THR_CASE(1);
  else if (nv == 2)
    FIER_THR_CASE(2);
  else
    FIER_THR_CASE(4);
#undef FIER_THR_CASE
  return hipGetLastError();
}

}  // namespace fier
