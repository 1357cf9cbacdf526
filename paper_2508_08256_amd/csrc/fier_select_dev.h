// Exact threshold selection among the candidates of the threshold bin: device functions of the threshold kernel
// (second kernel of the fused step).
#pragma once

#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

__device__ __forceinline__ float key_score(uint32_t key) {
  const uint32_t u = key ^ ((key >> 31) ? 0x80000000u : 0xffffffffu);
  return __uint_as_float(u);
}

// Candidates (key << 32 | token index) of threshold bin `tbin` sit in LDS; r_want >= 1 of them are to be selected,
// larger key first, equal keys by lower index.  One more histogram inside the bin (SUBBINS equal-width sub-bins),
// then the members of the decisive sub-bin are ranked pairwise.  On success T / idxT describe the last selected
// candidate and rsel[idx / 1024] has been incremented for every selected candidate; returns false (nothing
// modified in rsel) if the decisive sub-bin holds more than SUBMAX members.
// Every thread of the NT-thread workgroup must call it.  hist: SUBBINS words, sub_list: SUBMAX entries,
// scan_tmp: NT / 64 words, res: 2 words, n_sub: 1 word.
template <int NT, int SUBBINS, int SUBMAX>
__device__ __forceinline__ bool exact_select_lds(const unsigned long long* lcand, uint32_t n_cand, uint32_t r_want,
                                                 int tbin, float R, float scale, uint32_t* hist,
                                                 unsigned long long* sub_list, uint32_t* n_sub, uint32_t* res,
                                                 uint32_t* scan_tmp, uint32_t* rsel, uint32_t& T, int32_t& idxT) {
  static_assert(SUBBINS % NT == 0 || NT % SUBBINS == 0, "bins per thread");
  constexpr int PER = SUBBINS >= NT ? SUBBINS / NT : 1;
  const int tid = threadIdx.x;
  for (int k = tid; k < SUBBINS; k += NT) hist[k] = 0;
  if (tid == 0) *n_sub = 0;
  __syncthreads();
  const float lo_b = scale > 0.0f ? (float)tbin / scale - R : 0.0f;  // lower edge of the threshold bin
  const float scale2 = scale * (float)SUBBINS;
  for (uint32_t k = tid; k < n_cand; k += NT) {
    const float x = key_score((uint32_t)(lcand[k] >> 32));
    atomicAdd(&hist[sel_bin(x, -lo_b, scale2, SUBBINS)], 1u);
  }
  __syncthreads();
  // sub-bin t with (count in sub-bins > t) < r_want <= (count in sub-bins >= t); descending ownership
  {
    uint32_t cnt[PER], sum = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int bin = SUBBINS - 1 - (PER * tid + k);
      cnt[k] = bin >= 0 ? hist[bin] : 0;
      sum += cnt[k];
    }
    uint32_t total;
    uint32_t before = block_excl_scan_u32<NT / 64>(sum, scan_tmp, total);
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      if (before < r_want && r_want <= before + cnt[k]) {
        res[0] = (uint32_t)(SUBBINS - 1 - (PER * tid + k));
        res[1] = before;
      }
      before += cnt[k];
    }
    __syncthreads();
  }
  const int tsub = (int)res[0];
  const uint32_t r2 = r_want - res[1];  // rank wanted inside the sub-bin, 1-based
  const uint32_t n_in_sub = hist[tsub];
  __syncthreads();
  if (n_in_sub > (uint32_t)SUBMAX) return false;
  for (uint32_t k = tid; k < n_cand; k += NT) {
    const unsigned long long e = lcand[k];
    const int sb = sel_bin(key_score((uint32_t)(e >> 32)), -lo_b, scale2, SUBBINS);
    if (sb > tsub) atomicAdd(&rsel[(uint32_t)e / kRangeTokens], 1u);
    if (sb == tsub) sub_list[atomicAdd(n_sub, 1u)] = e;
  }
  __syncthreads();
  // rank the members of the decisive sub-bin: larger key first, equal keys by lower index
  for (uint32_t m = tid; m < n_in_sub; m += NT) {
    const unsigned long long me = sub_list[m];
    const uint32_t mk = (uint32_t)(me >> 32), mi = (uint32_t)me;
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n_in_sub; ++j) {
      const unsigned long long o = sub_list[j];
      const uint32_t ok = (uint32_t)(o >> 32), oi = (uint32_t)o;
      rank += (ok > mk) || (ok == mk && oi < mi);
    }
    if (rank < r2) atomicAdd(&rsel[mi / kRangeTokens], 1u);
    if (rank == r2 - 1) {
      res[0] = mk;
      res[1] = mi;
    }
  }
  __syncthreads();
  T = res[0];
  idxT = (int32_t)res[1];
  return true;
}

// The same selection streamed over all n scores of the unit (load(k) returns score k), restricted to the threshold
// bin: four 8-bit radix passes over the keys give T, an ordered pass gives idxT and the per-range counts of the
// selected candidates.  Slow (five passes by one workgroup) but independent of how the scores cluster.
// hist: 256 words; rsel may be null (no per-range counts wanted).  Every thread of the NT-thread workgroup must call it.
template <int NT, class Load>
__device__ __forceinline__ void stream_select(Load load, int n, int tbin, float R, float scale, uint32_t r_want,
                                              uint32_t* hist, uint32_t* scan_tmp, uint32_t* res, uint32_t* rsel,
                                              uint32_t& T, int32_t& idxT) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0, r = r_want;
#pragma unroll 1
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    for (int k = tid; k < 256; k += NT) hist[k] = 0;
    __syncthreads();
    for (int k = tid; k < n; k += NT) {
      const float x = load(k);
      const uint32_t key = score_key(x);
      if (sel_bin(x, R, scale, kSelBins) == tbin && (key & mask) == prefix)
        atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    // digit d with (count of digits > d) < r <= (count of digits >= d): thread t owns digit 255 - t
    const uint32_t cnt = tid < 256 ? hist[255 - tid] : 0;
    uint32_t total;
    const uint32_t before = block_excl_scan_u32<NT / 64>(cnt, scan_tmp, total);
    if (tid < 256 && before < r && r <= before + cnt) {
      res[0] = 255u - (uint32_t)tid;
      res[1] = before;
    }
    __syncthreads();
    prefix |= res[0] << shift;
    mask |= 0xffu << shift;
    r -= res[1];
    __syncthreads();
  }
  T = prefix;  // r = how many tokens with key == T (inside tbin) are selected: the lowest indices
  uint32_t run_eq = 0;
  for (int k0 = 0; k0 < n; k0 += NT) {
    const int k = k0 + tid;
    bool eq = false, gt = false;
    if (k < n) {
      const float x = load(k);
      const uint32_t key = score_key(x);
      const bool in_bin = sel_bin(x, R, scale, kSelBins) == tbin;
      eq = in_bin && key == T;
      gt = in_bin && key > T;
    }
    uint32_t total;
    const uint32_t before = run_eq + block_excl_scan_u32<NT / 64>(eq ? 1u : 0u, scan_tmp, total);
    if (rsel && (gt || (eq && before < r))) atomicAdd(&rsel[k / kRangeTokens], 1u);
    if (eq && before == r - 1) res[1] = (uint32_t)k;
    run_eq += total;
  }
  __syncthreads();
  idxT = (int32_t)res[1];
}

}  // namespace fier
