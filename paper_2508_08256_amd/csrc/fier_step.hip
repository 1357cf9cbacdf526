// Second kernel of the fused decode step: exact top-B threshold (Alg. 1 step 3) and attention over the selected
// rows (Alg. 1 step 4) in ONE launch, for grids whose workgroups are all resident at once.
//
// The score kernel has left, per unit, its scores and their 512-bin histogram over [-R, R].  Here a workgroup owns
// RPW consecutive 1024-token ranges of a unit and
//   1. finds, from the unit's histogram, the bin `tbin` that holds the B-th largest score (the same few hundred
//      integer additions in every workgroup of the unit: cheaper than a serial step somewhere plus the wait for it);
//   2. classifies its own scores: tokens in bins above tbin are selected for certain ("sure" rows, listed in LDS),
//      tokens inside tbin are the candidates for the threshold (about 1 % of the tokens), kept in LDS and published
//      as (key, index) pairs in the unit's candidate slots in memory;
//   3. counts its arrival.  One workgroup of the unit (the "selector": the unit's last workgroup, which as a rule
//      owns a partial range and few rows, once the others have arrived; whoever arrives last if that does not
//      happen within a bounded time) reads all candidates of the unit, histograms them once more inside the
//      threshold bin (1024 sub-bins), ranks the members of the decisive sub-bin pairwise (larger key first, equal
//      keys by lower index) and publishes the exact threshold (T, idxT) as one 64-bit word;
//   4. meanwhile every other workgroup attends over its sure rows (the selector after it has published): the bulk of
//      the gather runs while the serial selection is under way;
//   5. then picks up the threshold word (it is usually there by then; if not, the workgroup polls for a bounded
//      time), appends those of its candidates with `key > T or (key == T and index <= idxT)` to its row list and
//      attends over them too; stores its partial (m, l, o) per query head and counts a second arrival;
//   6. the unit's last arriver there merges the partials.
// A workgroup whose poll runs out says so in its partial (the sign of its l) and in the upper half of the second
// arrival counter; the merging workgroup then attends over that workgroup's threshold-bin rows itself before it
// merges.  The result therefore never depends on a poll
// succeeding, every wait is bounded and every wavefront exits.  A poll only ever lasts long when the unit's
// workgroups are not running together, which is why the launcher uses this kernel for resident grids and the
// three-kernel form (threshold kernel, then selection + attention) otherwise.
// All selection decisions are integer comparisons of order-preserving keys: exact and deterministic.
//
// The ascending index list of the selection (idx_out of the step, an optional output) is written by a small
// separate kernel from the scores and the threshold this kernel leaves in the unit's control block.
#include "fier_attn_dev.h"
#include "fier_dev.h"
#include "fier_kernels.h"
#include "fier_select_dev.h"

namespace fier {

namespace {

constexpr int kStepThreads = 256;
constexpr int kCandRegs = 8;        // candidate slots a selector thread holds in registers per sweep
constexpr int kCandLds = 256;       // candidates of a workgroup kept in LDS (the rest are read back from its slots)
constexpr int kMaxStepWgs = (1 << 20) / kRangeTokens;  // workgroups of one unit at most (max_ctx <= 2^20, RPW >= 1)
constexpr int kPollMax = 1 << 14;   // polls of the threshold word before a workgroup gives up (each >= 0.1 us)

// selector scratch in LDS (dead before the partials use the same bytes)
struct SelScratch {
  uint32_t hist[kSubBins];                    // sub-bin histogram; the radix fallback uses its first 256 words
  unsigned long long sub_list[kSubCandMax];   // members of the decisive sub-bin
  uint16_t seg_size[kMaxStepWgs];             // candidates published by each workgroup of the unit
  uint32_t res[2];
  uint32_t n_sub;
  uint32_t max_seg;
};

// The unit's threshold word: 0 = not there yet, else T << 32 | idxT + 2 (never zero: idxT >= -1).
__device__ __forceinline__ unsigned long long pack_threshold(uint32_t T, int32_t idxT) {
  return ((unsigned long long)T << 32) | (uint32_t)(idxT + 2);
}

// Exact threshold of a unit from the candidates its nc workgroups published: slot k * nc + w of ucand holds candidate
// k of workgroup w (k < useg[w], at most seg_cap per workgroup).  r_want >= 1 of the candidates are to be selected,
// larger key first, equal keys by lower index; T / idxT describe the last one selected.  One more histogram inside
// the threshold bin (kSubBins equal-width sub-bins), then the members of the decisive sub-bin are ranked pairwise.
// Returns false if a workgroup had more candidates than slots or the decisive sub-bin more than kSubCandMax members
// (the caller then falls back to the radix selection over the scores).  Every thread of the workgroup calls it.
__device__ __forceinline__ bool select_among_candidates(const unsigned long long* __restrict__ ucand,
                                                        const uint32_t* __restrict__ useg, int nc, uint32_t seg_cap,
                                                        uint32_t r_want, int tbin, float R, float hscale,
                                                        SelScratch* ss, uint32_t* scan_tmp, uint32_t& T,
                                                        int32_t& idxT) {
  const int tid = threadIdx.x;
  constexpr int kSegRegs = (kMaxStepWgs + kStepThreads - 1) / kStepThreads;
  // segment sizes and the first sweep of candidate slots leave together
  uint32_t my_max = 0;
  bool over = false;
  if (tid == 0) {
    ss->max_seg = 0;
    ss->res[0] = 0;
    ss->res[1] = 0;
    ss->n_sub = 0;
  }
  uint32_t segc[kSegRegs];
#pragma unroll
  for (int k = 0; k < kSegRegs; ++k) {
    const int w = k * kStepThreads + tid;
    segc[k] = w < nc ? load_coherent(&useg[w]) : 0u;
  }
  unsigned long long e[kCandRegs];
  const uint32_t slots_all = seg_cap * (uint32_t)nc;  // slots that exist for this unit's workgroups
#pragma unroll
  for (int k = 0; k < kCandRegs; ++k) {
    const uint32_t sidx = (uint32_t)(k * kStepThreads + tid);
    e[k] = sidx < slots_all ? load_coherent(&ucand[sidx]) : 0ull;
  }
#pragma unroll
  for (int k = 0; k < kSegRegs; ++k) {
    const int w = k * kStepThreads + tid;
    if (w < nc) {
      over = over || segc[k] > seg_cap;
      const uint32_t sz = segc[k] > seg_cap ? seg_cap : segc[k];
      ss->seg_size[w] = (uint16_t)sz;
      my_max = my_max > sz ? my_max : sz;
    }
  }
  for (int k = tid; k < kSubBins; k += kStepThreads) ss->hist[k] = 0;
  __syncthreads();
  if (my_max) atomicMax(&ss->max_seg, my_max);
  if (__syncthreads_or(over)) return false;
  // slots k * nc + w with k < max_seg may hold candidates: swept 8 x 256 at a time
  const uint32_t n_scan = ss->max_seg * (uint32_t)nc;
  const uint32_t sweep = (uint32_t)(kCandRegs * kStepThreads);
  const uint32_t n_sweeps = (n_scan + sweep - 1) / sweep;
  const float lo_b = hscale > 0.0f ? (float)tbin / hscale - R : 0.0f;  // lower edge of the threshold bin
  const float scale2 = hscale * (float)kSubBins;
  auto sub_of = [&](unsigned long long ent) {
    return sel_bin(key_score((uint32_t)(ent >> 32)), -lo_b, scale2, kSubBins);
  };
  // slot sidx = k * nc + w holds a candidate if k < seg_size[w]; a thread's slots are 256 apart, so (k, w) advance
  // by (256 / nc, 256 % nc) with a carry: no division per slot
  const uint32_t unc = (uint32_t)nc;
  const uint32_t step_k = (uint32_t)kStepThreads / unc, step_w = (uint32_t)kStepThreads % unc;
  uint32_t vmask = 0;  // first sweep: which of the thread's slots hold a candidate
  {
    uint32_t k_s = (uint32_t)tid / unc, w_s = (uint32_t)tid % unc;
    for (uint32_t sw = 0; sw < n_sweeps; ++sw) {
#pragma unroll
      for (int k = 0; k < kCandRegs; ++k) {
        const uint32_t sidx = sw * sweep + (uint32_t)(k * kStepThreads + tid);
        if (sw > 0) e[k] = sidx < n_scan ? load_coherent(&ucand[sidx]) : 0ull;
        const bool valid = sidx < n_scan && k_s < (uint32_t)ss->seg_size[w_s];
        if (valid) atomicAdd(&ss->hist[sub_of(e[k])], 1u);
        if (sw == 0 && valid) vmask |= 1u << k;
        k_s += step_k;
        w_s += step_w;
        if (w_s >= unc) {
          w_s -= unc;
          ++k_s;
        }
      }
    }
  }
  __syncthreads();
  // sub-bin t with (count in sub-bins > t) < r_want <= (count in sub-bins >= t); descending ownership
  {
    constexpr int PER = kSubBins / kStepThreads;
    uint32_t cntb[PER], sum = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      cntb[k] = ss->hist[kSubBins - 1 - (PER * tid + k)];
      sum += cntb[k];
    }
    uint32_t total;
    uint32_t before = block_excl_scan_u32<4>(sum, scan_tmp, total);
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      if (before < r_want && r_want <= before + cntb[k]) {
        ss->res[0] = (uint32_t)(kSubBins - 1 - (PER * tid + k));
        ss->res[1] = before;
      }
      before += cntb[k];
    }
    __syncthreads();
  }
  const int tsub = (int)ss->res[0];
  const uint32_t r2 = r_want - ss->res[1];  // rank wanted inside the sub-bin, 1-based
  const uint32_t n_in_sub = ss->hist[tsub];
  __syncthreads();
  if (n_in_sub > (uint32_t)kSubCandMax) return false;
  if (n_sweeps == 1) {  // the candidates are still in the registers
#pragma unroll
    for (int k = 0; k < kCandRegs; ++k)
      if ((vmask >> k & 1u) && sub_of(e[k]) == tsub) ss->sub_list[atomicAdd(&ss->n_sub, 1u)] = e[k];
  } else {
    uint32_t k_s = (uint32_t)tid / unc, w_s = (uint32_t)tid % unc;
    for (uint32_t sw = 0; sw < n_sweeps; ++sw) {
#pragma unroll
      for (int k = 0; k < kCandRegs; ++k) {
        const uint32_t sidx = sw * sweep + (uint32_t)(k * kStepThreads + tid);
        const bool valid = sidx < n_scan && k_s < (uint32_t)ss->seg_size[w_s];
        if (valid) {
          const unsigned long long ent = load_coherent(&ucand[sidx]);
          if (sub_of(ent) == tsub) ss->sub_list[atomicAdd(&ss->n_sub, 1u)] = ent;
        }
        k_s += step_k;
        w_s += step_w;
        if (w_s >= unc) {
          w_s -= unc;
          ++k_s;
        }
      }
    }
  }
  __syncthreads();
  // rank the members of the decisive sub-bin: larger key first, equal keys by lower index
  for (uint32_t m = tid; m < n_in_sub; m += kStepThreads) {
    const unsigned long long me = ss->sub_list[m];
    const uint32_t mk = (uint32_t)(me >> 32), mi = (uint32_t)me;
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n_in_sub; ++j) {
      const unsigned long long o = ss->sub_list[j];
      const uint32_t ok = (uint32_t)(o >> 32), oi = (uint32_t)o;
      rank += (ok > mk) || (ok == mk && oi < mi);
    }
    if (rank == r2 - 1) {
      ss->res[0] = mk;
      ss->res[1] = mi;
    }
  }
  __syncthreads();
  T = ss->res[0];
  idxT = (int32_t)ss->res[1];
  return true;
}

}  // namespace

// What the kernel needs besides the template parameters; passed by value.
struct StepArgs {
  const float* scores;
  UnitCtl* ctl;
  uint32_t* ghist;
  const int32_t* budgets;
  int max_budget;
  unsigned long long* cand;  // [units][cand_pitch]: slot k * nc + w = k-th candidate of workgroup w of the unit
  uint32_t* sel_cnt;         // [units][wgs_per_unit]: rows each workgroup ended up with (for the index-list kernel)
  uint32_t* seg_cnt;         // [units][wgs_per_unit]
  const uint4* K;
  const uint4* V;
  const uint4* q;
  const int32_t* seq_lens;
  int extra;
  float scale_log2e;
  float* po;
  float* pm;
  float* pl;
  float* out;
  int32_t* count_out;
  float* kabsmax;
  const float* newmax;
  int n_kv_heads, max_ctx, order, wgs_per_unit;
  size_t cand_pitch;
  int flags;  // tests: bit 0 = no workgroup picks up the threshold (the merging workgroup attends over all
              // threshold-bin rows); bit 1 = checksums of the attended rows
  KvLayout lay;
};

// LDS of one workgroup of the step's second kernel
template <int NREP, int RPW>
struct StepLds {
  static constexpr size_t kScratchBytes =
      sizeof(SelScratch) > sizeof(float) * NREP * kPartialFloats ? sizeof(SelScratch) : sizeof(float) * NREP * kPartialFloats;
  static_assert(kScratchBytes >= sizeof(float) * 4 * 130, "merge_heads needs 4 x 130 floats");
  __attribute__((aligned(16))) unsigned char scratch[kScratchBytes];  // selector scratch, then partial staging
  uint16_t rows[kRangeTokens * RPW];  // the rows to attend over (offsets from tok0): sure rows, then selected candidates
  uint16_t coff[kCandLds];            // the workgroup's first candidates: offsets from tok0 ...
  uint32_t ckey[kCandLds];            // ... and keys
  uint32_t scan_tmp[4];
  int found[2];
  uint32_t flag;
  unsigned long long thr_sh;
  int32_t lblk[RPW * kRangeTokens / 64];  // paged rows: block numbers of this workgroup's tokens
};

// Workgroup `wg` of unit `unit`.
template <int DT, int NREP, int RPW, bool STREAM>
__device__ __forceinline__ void step_attend_body(const StepArgs& a, const int unit, const int wg,
                                                 StepLds<NREP, RPW>& lds) {
  constexpr int CAP = kRangeTokens * RPW;  // tokens the workgroup owns
  constexpr int SEGCAP = CAP / 4;          // candidates it can publish (a quarter of its tokens)
  uint16_t* const rows = lds.rows;
  uint16_t* const coff = lds.coff;
  uint32_t* const ckey = lds.ckey;
  uint32_t* const scan_tmp = lds.scan_tmp;
  int* const found = lds.found;
  uint32_t& flag = lds.flag;
  unsigned long long& thr_sh = lds.thr_sh;
  int32_t* const lblk = lds.lblk;
  float* const sh_o = reinterpret_cast<float*>(lds.scratch);
  SelScratch* const ss = reinterpret_cast<SelScratch*>(lds.scratch);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int cn = tid & 15;
  const int max_ctx = a.max_ctx;
  const int b = unit / a.n_kv_heads;
  UnitCtl* __restrict__ c = &a.ctl[unit];
  uint32_t* __restrict__ gh = a.ghist + (size_t)unit * kSelBins;
  // what does not depend on the sequence length leaves with it: the unit's histogram (thread t owns bins 511 - 2t
  // and 510 - 2t: descending score order), the range of the binning, the budget
  const uint2 hpair = *reinterpret_cast<const uint2*>(gh + (kSelBins - 2 - 2 * tid));
  const float R = c->R, hscale = c->scale;
  int B = a.budgets[b];
  int n = a.seq_lens[b] + a.extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  const int tok0 = wg * CAP;
  if (tok0 >= n && wg != 0) return;
  const int nc = n > 0 ? (n + CAP - 1) / CAP : 1;  // workgroups of this unit that run
  FIER_PROF_WG(2)
  const int n_slots = a.wgs_per_unit + 1;          // partial slots per (unit, head): one spare for the merger

  const KvRows kv = a.lay.rows_of(unit);
  if (kv.blocks && tid < RPW * kRangeTokens / 64) {  // in flight during the selection; barriers follow
    const int bi = (tok0 >> kv.shift) + tid;
    lblk[tid] = bi < a.lay.blocks_per_seq ? kv.blocks[bi] : 0;
  }
  const float* __restrict__ s_unit = a.scores + (size_t)unit * max_ctx;
  unsigned long long* __restrict__ ucand = a.cand + (size_t)unit * a.cand_pitch;
  uint32_t* __restrict__ useg = a.seg_cnt + (size_t)unit * a.wgs_per_unit;
  uint32_t* __restrict__ usel = a.sel_cnt + (size_t)unit * a.wgs_per_unit;

  // ---- 1. the workgroup's scores; meanwhile the threshold bin from the histogram ---------------------------------
  float4 v[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    // i + 3 < max_ctx; entries >= n are masked below.  A thread past the end loads the unit's first scores instead of
    // branching round the load: with branches the compiler cannot count the loads in flight and waits for all of them
    // before the histogram scan below, which needs none of them
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    v[rr] = *reinterpret_cast<const float4*>(s_unit + (i < n ? i : 0));
  }
  B = B > a.max_budget ? a.max_budget : B;
  B = B > n ? n : B;
  B = B < 0 ? 0 : B;
  if (tid == 0) {
    found[0] = B >= n ? -1 : kSelBins;  // everything / nothing selected by bin alone
    found[1] = 0;
  }
  {
    uint32_t total;
    const uint32_t c0 = hpair.y, c1 = hpair.x;
    const uint32_t before = block_excl_scan_u32<4>(c0 + c1, scan_tmp, total);  // has barriers
    if (B > 0 && B < n) {
      if (before < (uint32_t)B && (uint32_t)B <= before + c0) {
        found[0] = kSelBins - 1 - 2 * tid;
        found[1] = (int)before;
      } else if (before + c0 < (uint32_t)B && (uint32_t)B <= before + c0 + c1) {
        found[0] = kSelBins - 2 - 2 * tid;
        found[1] = (int)(before + c0);
      }
    }
    __syncthreads();
  }
  const int tbin = found[0];
  const uint32_t above = (uint32_t)found[1];
  const bool need_threshold = tbin >= 0 && tbin < kSelBins && B > 0;

  // ---- 2. classify the workgroup's tokens: sure rows and candidates ------------------------------------------------
  uint32_t dmask = 0, cmask = 0;  // bit 4 rr + j = token j of the thread in range rr
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    const float vv[4] = {v[rr].x, v[rr].y, v[rr].z, v[rr].w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool ok = i + j < n;
      const int bin = sel_bin(vv[j], R, hscale, kSelBins);
      dmask |= (ok && bin > tbin) ? 1u << (4 * rr + j) : 0u;
      cmask |= (ok && bin == tbin) ? 1u << (4 * rr + j) : 0u;
    }
  }
  uint32_t listed;  // sure rows (low half) and candidates (high half) of the whole workgroup
  {
    // list positions in thread order (one workgroup scan for both lists), so that the lists, and with them the order
    // in which the rows are summed, are the same in every run
    const uint32_t packed = (uint32_t)__builtin_popcount(dmask) | ((uint32_t)__builtin_popcount(cmask) << 16);
    const uint32_t at = block_excl_scan_u32<4>(packed, scan_tmp, listed);
    uint32_t pd = at & 0xffffu, pc = at >> 16;
    if constexpr (RPW >= 2) {
      // the few tokens of a thread that are listed, by their bits (ascending bit = ascending token): a thread holds
      // 4 RPW tokens of which a few per cent are selected, so walking the set bits beats 4 RPW predicated blocks
      // (measured: 1.9 us of 67 at 8 ranges per workgroup, 0.3 of 34.5 at two; with one range the blocks are faster)
      for (uint32_t m = dmask; m; m &= m - 1u) {
        const uint32_t bit = (uint32_t)__builtin_ctz(m);
        rows[pd++] = (uint16_t)((bit >> 2) * (uint32_t)kRangeTokens + 4u * (uint32_t)tid + (bit & 3u));
      }
      for (uint32_t m = cmask; m; m &= m - 1u) {
        const uint32_t bit = (uint32_t)__builtin_ctz(m);
        float x = 0.f;  // the token's score, picked from the registers without indexing them
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
          x = bit == 4u * rr ? v[rr].x : x;
          x = bit == 4u * rr + 1u ? v[rr].y : x;
          x = bit == 4u * rr + 2u ? v[rr].z : x;
          x = bit == 4u * rr + 3u ? v[rr].w : x;
        }
        const uint32_t off = (bit >> 2) * (uint32_t)kRangeTokens + 4u * (uint32_t)tid + (bit & 3u);
        const uint32_t key = score_key(x);
        if (pc < (uint32_t)kCandLds) {
          coff[pc] = (uint16_t)off;
          ckey[pc] = key;
        }
        if (pc < (uint32_t)SEGCAP)
          store_coherent(&ucand[(size_t)pc * nc + wg], ((unsigned long long)key << 32) | (uint32_t)(tok0 + (int)off));
        ++pc;
      }
    } else {
#pragma unroll
      for (int rr = 0; rr < RPW; ++rr) {
        const float vv[4] = {v[rr].x, v[rr].y, v[rr].z, v[rr].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t off = (uint32_t)(rr * kRangeTokens + 4 * tid + j);
          if (dmask >> (4 * rr + j) & 1u) rows[pd++] = (uint16_t)off;
          if (cmask >> (4 * rr + j) & 1u) {
            const uint32_t key = score_key(vv[j]);
            if (pc < (uint32_t)kCandLds) {
              coff[pc] = (uint16_t)off;
              ckey[pc] = key;
            }
            if (pc < (uint32_t)SEGCAP)
              store_coherent(&ucand[(size_t)pc * nc + wg], ((unsigned long long)key << 32) | (uint32_t)(tok0 + (int)off));
            ++pc;
          }
        }
      }
    }
  }
  int n_rows = (int)(listed & 0xffffu);
  const int n_cand = (int)(listed >> 16);
  uint32_t chk_sum = 0;  // (tests) sum of the token indices this thread put on the list

  // ---- 3. the exact threshold, found by the unit's last arriver ------------------------------------------------------
  uint4 qr[NREP];
#pragma unroll
  for (int h = 0; h < NREP; ++h) qr[h] = a.q[((size_t)unit * NREP + h) * (kD / 8) + cn];
  const uint4* q_unit = a.q + (size_t)unit * NREP * (kD / 8);
  AttnState<NREP> st;
  st.init();
  const int first_block = tok0 >> kv.shift;
  auto row_own = [&](int j) {
    const int t = tok0 + (int)rows[j];
    return kv.blocks ? (size_t)lblk[(t >> kv.shift) - first_block] * kv.block_stride + kv.base + (size_t)(t & kv.mask)
                     : kv.base + (size_t)t;
  };
  auto attend_own = [&](int from, int to, bool resume) {
    if constexpr (NREP >= 3)
      attend_rows_mfma<DT, NREP, false, false, STREAM>(a.K, a.V, q_unit, row_own, from, to, a.scale_log2e, st, sh_o, resume);
    else
      attend_rows<DT, NREP, false, STREAM>(a.K, a.V, qr, row_own, from, to, a.scale_log2e, st);
  };
  bool picked = true;  // the workgroup's threshold-bin rows are on its list (or it has none)
  uint32_t T = 0;
  int32_t idxT = -1;
  bool have = false;
  if (need_threshold) {
    if (tid == 0) store_coherent(&useg[wg], (uint32_t)n_cand);
    // The selector attends over its own rows only after it has published the threshold, so it should be a workgroup
    // with few rows: the unit's last workgroup (a partial range as a rule) holds its arrival back until the nc - 1
    // others have arrived and then selects without counting itself.  It waits for a bounded time; if that runs out it
    // arrives like the others and whoever then arrives last selects.
    bool selects = false;
    if (wg == nc - 1 && nc > 1) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this workgroup's candidates have been acknowledged
      if (tid == 0) {
        uint32_t arrived = 0;
        for (int spin = 0; spin < kPollMax; ++spin) {
          arrived = load_coherent(&c->arrive[1]);
          if (arrived >= (uint32_t)(nc - 1)) break;
          __builtin_amdgcn_s_sleep(2);
        }
        flag = arrived >= (uint32_t)(nc - 1) ? 1u : 0u;
      }
      __syncthreads();
      selects = flag != 0u;
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      asm volatile("" ::: "memory");
      if (!selects) selects = last_arriver(&c->arrive[1], (uint32_t)nc, &flag);
    } else {
      selects = last_arriver(&c->arrive[1], (uint32_t)nc, &flag);
    }
    if (selects) {
      FIER_PROF(13, unit == 0)
      __builtin_amdgcn_s_setprio(3);
      if (!select_among_candidates(ucand, useg, nc, (uint32_t)SEGCAP, (uint32_t)B - above, tbin, R, hscale, ss, scan_tmp,
                                   T, idxT)) {
        // candidates that do not fit (scores clustered far more tightly than the a-priori range resolves): radix
        // selection streamed over the unit's scores
        __syncthreads();
        stream_select<kStepThreads>([&](int k) { return s_unit[k]; }, n, tbin, R, hscale, (uint32_t)B - above, ss->hist,
                                    scan_tmp, ss->res, nullptr, T, idxT);
      }
      if (tid == 0) {
        store_coherent(&c->thr, pack_threshold(T, idxT));
        c->arrive[1] = 0;
      }
      __builtin_amdgcn_s_setprio(0);
      have = true;
      __syncthreads();  // the scratch is reused below
      FIER_PROF(15, unit == 0)
    }
  } else {
    __syncthreads();  // the row list is complete
  }
  FIER_PROF_WG(3)
  // ---- 4. attention over the sure rows, while the unit's threshold is being found ----------------------------------
  attend_own(0, n_rows, false);
  const int n_sure = n_rows;
  FIER_PROF_WG(4)
  // ---- 5. the threshold is picked up; the selected candidates join the row list -----------------------------------
  if (need_threshold) {
    if (!have && n_cand > 0 && n_cand <= SEGCAP) {
      __syncthreads();
      if (tid == 0) {
        unsigned long long w = 0;
        for (int spin = 0; spin < kPollMax; ++spin) {
          w = load_coherent(&c->thr);
          if (w) break;
          __builtin_amdgcn_s_sleep(4);
        }
        thr_sh = w;
      }
      __syncthreads();
      const unsigned long long w = thr_sh;
      have = w != 0ull;
      T = (uint32_t)(w >> 32);
      idxT = (int32_t)(uint32_t)w - 2;
    }
    picked = n_cand == 0;
    if (have && n_cand > 0 && n_cand <= SEGCAP && !(a.flags & 1)) {
      __syncthreads();  // every wavefront is done with the rows listed so far
      // in candidate (= token) order
      for (int k0 = 0; k0 < n_cand; k0 += kStepThreads) {
        const int k = k0 + tid;
        bool sel = false;
        uint32_t off = 0;
        if (k < n_cand) {
          uint32_t key;
          if (k < kCandLds) {
            off = coff[k];
            key = ckey[k];
          } else {  // the workgroup's own slot
            const unsigned long long ent = load_coherent(&ucand[(size_t)k * nc + wg]);
            key = (uint32_t)(ent >> 32);
            off = (uint32_t)ent - (uint32_t)tok0;
          }
          sel = key > T || (key == T && tok0 + (int)off <= idxT);
        }
        uint32_t n_sel;
        const uint32_t at = block_excl_scan_u32<4>(sel ? 1u : 0u, scan_tmp, n_sel);
        if (sel) rows[n_rows + (int)at] = (uint16_t)off;
        n_rows += (int)n_sel;
      }
      picked = true;
    }
    __syncthreads();  // the row list is complete
  }
  if (tid == 0) store_coherent(&usel[wg], (uint32_t)n_rows);  // the merging workgroup may add to it
  attend_own(n_sure, n_rows, true);
  FIER_PROF_WG(5)
  if (a.flags & 2) {
    for (int j = tid; j < n_rows; j += kStepThreads) chk_sum += (uint32_t)(tok0 + (int)rows[j]);
    chk_sum = wave_sum_u32(chk_sum);
    if (lane == 0 && chk_sum) atomicAdd(&c->chk_sum, chk_sum);
    if (tid == 0 && n_rows) atomicAdd(&c->chk_cnt, (uint32_t)n_rows);
  }
  // a partial that lacks the workgroup's threshold-bin rows is marked as such (the sign of its l), and the workgroup
  // counts itself in the upper half of the arrival counter: the merging workgroup learns from the counter's value,
  // without loading anything, whether there are such rows
  store_partials<NREP, true>(st, sh_o, unit, n_slots, wg, a.po, a.pm, a.pl, !picked);
  FIER_PROF_WG(6)

  const uint32_t before = arrive_add(&c->arrive[2], picked ? 1u : 0x10001u, &flag);
  if ((before & 0xffffu) != (uint32_t)nc - 1u) return;
  // ---- the unit's last workgroup: anything left over, then the merge ----------------------------------------------
  int n_used = nc;
  if (need_threshold) {
    if (!have) {  // published before its writer's second arrival; in flight together with the partials
      const unsigned long long wthr = load_coherent(&c->thr);
      T = (uint32_t)(wthr >> 32);
      idxT = (int32_t)(uint32_t)wthr - 2;
    }
    if ((before >> 16) != 0u || !picked) {  // the same in every thread
      // Some workgroup did not put its threshold-bin rows on its list: they are attended over here, 256 candidates
      // at a time through the row list (this workgroup's own rows are done), into the spare partial slot.
      for (int w = tid; w < nc; w += kStepThreads)
        ss->seg_size[w] = load_coherent(&a.pl[(size_t)unit * NREP * n_slots + w]) < 0.f ? 1 : 0;  // head 0's slots
      __syncthreads();
      st.init();
      bool resumed = false;
      uint32_t cnt_x = 0, sum_x = 0;
      for (int w = 0; w < nc; ++w) {
        if (!ss->seg_size[w]) continue;  // the same in every thread
        const int base = w * CAP;
        const int span = n - base < CAP ? n - base : CAP;
        const uint32_t cnt_before = cnt_x;
        for (int k0 = 0; k0 < span; k0 += kStepThreads) {
          const int t = base + k0 + tid;
          bool sel = false;
          if (k0 + tid < span) {
            const float x = s_unit[t];
            const uint32_t key = score_key(x);
            sel = sel_bin(x, R, hscale, kSelBins) == tbin && (key > T || (key == T && t <= idxT));
          }
          uint32_t n_x;
          const uint32_t at = block_excl_scan_u32<4>(sel ? 1u : 0u, scan_tmp, n_x);  // its first barrier frees the list
          if (sel) {
            rows[at] = (uint16_t)(k0 + tid);
            sum_x += (uint32_t)t;
          }
          __syncthreads();
          auto row_any = [&](int j) { return kv.row(base + (int)rows[j]); };
          if constexpr (NREP >= 3)
            attend_rows_mfma<DT, NREP, false, false, STREAM>(a.K, a.V, q_unit, row_any, 0, (int)n_x, a.scale_log2e, st, sh_o,
                                                             resumed);
          else
            attend_rows<DT, NREP, false, STREAM>(a.K, a.V, qr, row_any, 0, (int)n_x, a.scale_log2e, st);
          resumed = true;
          cnt_x += n_x;
        }
        // that workgroup's row count, for the index-list kernel (it arrived long ago: its own store is there)
        if (tid == 0) store_coherent(&usel[w], load_coherent(&usel[w]) + (cnt_x - cnt_before));
      }
      if (a.flags & 2) {
        sum_x = wave_sum_u32(sum_x);
        if (lane == 0 && sum_x) atomicAdd(&c->chk_sum, sum_x);
        if (tid == 0 && cnt_x) atomicAdd(&c->chk_cnt, cnt_x);
      }
      store_partials<NREP, true>(st, sh_o, unit, n_slots, nc, a.po, a.pm, a.pl);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the spare slot is read back below by other wavefronts
      __syncthreads();
      n_used = nc + 1;
    }
  }
  merge_heads<NREP>(a.po, a.pm, a.pl, unit, n_slots, n_used, sh_o, a.out + (size_t)unit * NREP * kD);
  FIER_PROF_WG(7)
  // counters back to zero for the next call, the unit's histogram too (all its readers have arrived); the
  // selection for the index-list kernel
  for (int k = tid; k < kSelBins; k += kStepThreads) gh[k] = 0;
  if (tid == 0) {
    c->arrive[2] = 0;
    c->thr = 0ull;
    c->tbin = tbin;
    c->above = above;
    c->budget = B;
    c->T = T;
    c->idxT = idxT;
    if (a.count_out) a.count_out[unit] = B;
  }
  // the step appended a row: fold the bound of its re-quantized group into the unit's per-channel bound
  if (a.extra && a.seq_lens[b] < max_ctx && tid < kD) {
    float* slot = a.kabsmax + (size_t)unit * kD + tid;
    const float nm = a.newmax[(size_t)unit * kD + tid];
    if (nm > *slot) *slot = nm;
  }
}

// order: 0 = grid (workgroups, units); 1 = grid (units, workgroups); 2 = one-dimensional, groups of 8 units, a
// group's workgroups together and unit % 8 fastest (see the launcher)
__device__ __forceinline__ void step_unit_wg(const StepArgs& a, int id_x, int id_y, int& unit, int& wg) {
  if (a.order == 2) {
    const int g = id_x / (8 * a.wgs_per_unit);
    const int rem = id_x - g * 8 * a.wgs_per_unit;
    wg = rem >> 3;
    unit = 8 * g + (rem & 7);
  } else {
    unit = a.order ? id_x : id_y;
    wg = a.order ? id_y : id_x;
  }
}

// grid: wgs_per_unit workgroups per unit (dispatch order given by `order`), block 256.
// (the second launch bound asks the compiler for the registers-per-thread that let 5 / 4 / 3 / 2 workgroups share a
// CU: the gather wants many rows in flight per CU more than it wants registers -- but not at the price of spills:
// with 4 query heads per kv head a bound of 4 left 60 bytes of scratch per lane and cost 3 to 5 us per step)
constexpr int step_wgs_per_cu(int n_rep) { return n_rep <= 2 ? 5 : (n_rep <= 3 ? 4 : (n_rep <= 5 ? 3 : 2)); }
// STREAM: the gathered rows are loaded with the streaming hint (with three or more query heads per kv head, where
// the K rows go to the matrix cores in four pieces per row, the V rows only).
template <int DT, int NREP, int RPW, bool STREAM>
__global__ __launch_bounds__(kStepThreads, step_wgs_per_cu(NREP)) void step_attend_kernel(
    const StepArgs a) {
  __shared__ StepLds<NREP, RPW> lds;
  int unit, wg;
  step_unit_wg(a, (int)blockIdx.x, (int)blockIdx.y, unit, wg);
  step_attend_body<DT, NREP, RPW, STREAM>(a, unit, wg, lds);
}

// The ascending index list of the step's selection: idx[unit][0 .. budget) from the scores, the threshold the step
// left in the control block and the row count every workgroup of the step's second kernel recorded.  grid (units,
// workgroups per unit), block 256: workgroup (unit, wg) covers the same rpw 1024-token ranges as workgroup wg of the
// step, starts its part of the list at the sum of the counts of the workgroups before it and fills it in token
// order.  An optional output of the step, off its fast path.
template <int RPW>
__global__ __launch_bounds__(kStepThreads) void step_emit_idx_kernel(const float* __restrict__ scores,
                                                                     const int32_t* __restrict__ seq_lens, int extra,
                                                                     const UnitCtl* __restrict__ ctl,
                                                                     const uint32_t* __restrict__ sel_cnt,
                                                                     int wgs_per_unit, int max_budget,
                                                                     int32_t* __restrict__ idx, int n_kv_heads,
                                                                     int max_ctx) {
  __shared__ uint32_t wtot[RPW + 1][4];  // per wavefront: selected tokens of each range, rows of the workgroups before
  const int unit = blockIdx.x, wg = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int n = seq_lens[unit / n_kv_heads] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  const int tok0 = wg * RPW * kRangeTokens;
  if (tok0 >= n) return;
  const float* __restrict__ s = scores + (size_t)unit * max_ctx;
  // this workgroup's scores, the counts of the workgroups before it and the unit's threshold leave together
  float4 v[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    v[rr] = *reinterpret_cast<const float4*>(s + (i < n ? i : 0));  // i + 3 < max_ctx; masked below
  }
  uint32_t mine = 0;
  for (int w = tid; w < wg; w += kStepThreads) mine += sel_cnt[(size_t)unit * wgs_per_unit + w];
  const UnitCtl* __restrict__ c = &ctl[unit];
  const int tbin = c->tbin;
  const float R = c->R, scale = c->scale;
  const uint32_t T = c->T;
  const int32_t idxT = c->idxT;
  // all ranges' positions with one barrier: per range a scan inside the wavefront, the wavefronts' totals through LDS
  uint32_t selm[RPW], incl[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    const float vv[4] = {v[rr].x, v[rr].y, v[rr].z, v[rr].w};
    selm[rr] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int bin = sel_bin(vv[j], R, scale, kSelBins);
      const uint32_t key = score_key(vv[j]);
      const bool sel =
          i + j < n && (bin > tbin || (bin == tbin && (key > T || (key == T && i + j <= idxT))));
      selm[rr] |= sel ? 1u << j : 0u;
    }
    incl[rr] = wave_incl_scan_u32((uint32_t)__builtin_popcount(selm[rr]), lane);
  }
  const uint32_t mine_w = wave_sum_u32(mine);
  if (lane == 63) {
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) wtot[rr][wave] = incl[rr];
    wtot[RPW][wave] = mine_w;
  }
  __syncthreads();
  uint32_t run = wtot[RPW][0] + wtot[RPW][1] + wtot[RPW][2] + wtot[RPW][3];  // the list position of this workgroup's first row
  int32_t* __restrict__ out = idx + (size_t)unit * max_budget;
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const uint32_t t0 = wtot[rr][0], t1 = wtot[rr][1], t2 = wtot[rr][2], t3 = wtot[rr][3];
    const uint32_t wave_off = (wave > 0 ? t0 : 0u) + (wave > 1 ? t1 : 0u) + (wave > 2 ? t2 : 0u);
    uint32_t pos = run + wave_off + incl[rr] - (uint32_t)__builtin_popcount(selm[rr]);
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (selm[rr] >> j & 1u) {
        if (pos < (uint32_t)max_budget) out[pos] = i + j;
        ++pos;
      }
    run += t0 + t1 + t2 + t3;
  }
}

// Workgroups of the step's second kernel that a 256-CU chip holds at once (the kernel's second launch bound).
static long step_resident_wgs(int n_rep) { return 256L * step_wgs_per_cu(n_rep); }

// Ranges per workgroup of the one-launch form (rows per 1024-token range = 1024 * budget / context):
//   * at least 96 selected rows per workgroup;
//   * more where fewer, larger workgroups make the grid resident at once;
//   * and twice as many where that still leaves two workgroups per CU and at most 288 rows per workgroup.  Measured
//     (us per step): 32 units x 32k, 112 rows per range: 35.0 with one range per workgroup, 34.0 with two, 38.1 with
//     four; 32 units x 16k (two ranges = one workgroup per CU): 25.8 / 27.4; 32 units x 64k, B = 7209: 50.9 with two
//     ranges (225 rows), 51.5 with four; 64 units x 32k: 50.6 with two, 51.9 with four.
int step_ranges_per_wg(int units, int n_rep, int max_budget, int max_ctx) {
  const double per_range = 1024.0 * (double)max_budget / (double)max_ctx;
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  auto wgs = [&](int r) { return (long)units * ((n_ranges + r - 1) / r); };
  int rpw = 1;
  while (rpw < 8 && per_range * rpw < 96.0) rpw *= 2;
  while (rpw < 8 && wgs(rpw) > step_resident_wgs(n_rep)) rpw *= 2;
  if (rpw < 8 && per_range * (2 * rpw) <= 288.0 && wgs(2 * rpw) >= 512) rpw *= 2;
  return rpw;
}

static bool fill_step_args(StepArgs& a, int rpw, int order, KvLayout lay, const StepBuffers& sb, const void* K,
                           const void* V, const void* q, const int32_t* seq_lens, int extra, const int32_t* budgets,
                           int max_budget, float sm_scale, int32_t* count_out, float* out, float* kabsmax, int units,
                           int n_kv_heads, int max_ctx, int flags) {
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const int n_wgs = (n_ranges + rpw - 1) / rpw;
  a.scores = sb.scores;
  a.ctl = sb.ctl;
  a.ghist = sb.hist;
  a.budgets = budgets;
  a.max_budget = max_budget;
  a.cand = sb.cand;
  a.seg_cnt = sb.seg_cnt;
  a.sel_cnt = sb.sel_cnt;
  a.K = (const uint4*)K;
  a.V = (const uint4*)V;
  a.q = (const uint4*)q;
  a.seq_lens = seq_lens;
  a.extra = extra;
  a.scale_log2e = sm_scale * 1.4426950408889634f;
  a.po = sb.po;
  a.pm = sb.pm;
  a.pl = sb.pl;
  a.out = out;
  a.count_out = count_out;
  a.kabsmax = kabsmax;
  a.newmax = sb.newmax;
  a.n_kv_heads = n_kv_heads;
  a.max_ctx = max_ctx;
  a.order = order;
  a.wgs_per_unit = n_wgs;
  a.cand_pitch = sb.cand_pitch;
  a.flags = flags;
  a.lay = lay;
  return (size_t)n_wgs * (rpw * kRangeTokens / 4) <= sb.cand_pitch && n_wgs <= sb.seg_pitch;
}

template <int DT, int RPW>
static hipError_t launch_step_attend_dt(KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                        const void* q, const int32_t* seq_lens, int extra, const int32_t* budgets,
                                        int max_budget, float sm_scale, int32_t* count_out, float* out, float* kabsmax,
                                        int units, int n_kv_heads, int max_ctx, int flags, hipStream_t st) {
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const int n_wgs = (n_ranges + RPW - 1) / RPW;
  // Dispatch order.  Workgroups go round-robin to the 8 XCDs in the order of their linear index; when a unit's
  // workgroups all run on one XCD, its scores, candidates, partials and arrival counters stay in that XCD's L2.
  //   1: units fastest (a multiple of 8 units puts unit u on XCD u % 8), for grids that are resident at once;
  //   2: longer grids with a multiple of 8 units: groups of 8 units one after the other, inside a group the
  //      workgroups in range order and unit % 8 fastest -- the same XCD assignment, but a unit's workgroups stay
  //      together in time, which also keeps the wait for the unit's threshold short;
  //   0: ranges fastest, otherwise.
  // Order 1 only while every workgroup is resident at once (the second launch bound of the kernel: 5 / 4 / 3 / 2
  // workgroups per CU, 256 CUs): its workgroups poll for their unit's threshold, and a unit spread over two rounds
  // of workgroups would have the first round waiting for the second.
  const long resident = step_resident_wgs(n_rep);
  const int order = (long)units * n_wgs <= resident ? 1 : (units % 8 == 0 ? 2 : 0);
  dim3 grid = order == 2 ? dim3((unsigned)units * (unsigned)n_wgs) : (order ? dim3(units, n_wgs) : dim3(n_wgs, units));
  StepArgs a;
  if (!fill_step_args(a, RPW, order, lay, sb, K, V, q, seq_lens, extra, budgets, max_budget, sm_scale, count_out, out,
                      kabsmax, units, n_kv_heads, max_ctx, flags))
    return hipErrorInvalidValue;
  // The streaming hint on the gathered K / V rows (they are read once and leave the caches to the scores, candidates
  // and partials).  Measured with the step rotating over 12 layer caches, us per step without / with the hint here
  // and on the score kernel's loads: 32 units x 32k 33.5 / 32.95 (this kernel alone 22.7 / 21.3), 32 x 64k at
  // B = 16384 76.8 / 72.3 (59.0 / 53.2), at B = 256 32.6 / 31.9; 8 units x 4k, whose rows the caches hold, lost 0.9 us
  // with it.  Hence from 8 MB of gathered rows per launch.  (Rotating over 3 to 6 caches overstates the gain: 2 us
  // at 32 x 32k.)  The matrix-core gather (3 or more heads per kv head) lost by it on the K rows, which it loads in
  // four pieces per row (32 units x 128k +0.6 us, the ragged 128-unit batch +4), and gains on the V rows alone:
  // 32 x 128k 61.5 / 59.7, the ragged batch 101.3 / 100.8.
  const bool stream = (long)units * max_budget * (2 * kD * 2) >= (8L << 20);
#define FIER_STEP_CASE_S(R)                                                       \
  case R:                                                                         \
    if (stream) step_attend_kernel<DT, R, RPW, true><<<grid, kStepThreads, 0, st>>>(a);  \
    else step_attend_kernel<DT, R, RPW, false><<<grid, kStepThreads, 0, st>>>(a); \
    break;
  switch (n_rep) {
    FIER_STEP_CASE_S(1)
    FIER_STEP_CASE_S(2)
    FIER_STEP_CASE_S(3)
    FIER_STEP_CASE_S(4)
    FIER_STEP_CASE_S(5)
    FIER_STEP_CASE_S(6)
    FIER_STEP_CASE_S(7)
    FIER_STEP_CASE_S(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_STEP_CASE_S
  return hipGetLastError();
}

hipError_t launch_step_attend(int dtype, KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                              const void* q, const int32_t* seq_lens, int extra, const int32_t* budgets, int max_budget,
                              float sm_scale, int32_t* count_out, float* out, float* kabsmax, int units, int n_kv_heads,
                              int max_ctx, int flags, hipStream_t st) {
#define FIER_STEP_RPW(DT, RPW)                                                                                        \
  return launch_step_attend_dt<DT, RPW>(lay, n_rep, sb, K, V, q, seq_lens, extra, budgets, max_budget, sm_scale,      \
                                        count_out, out, kabsmax, units, n_kv_heads, max_ctx, flags, st)
  const int rpw = step_ranges_per_wg(units, n_rep, max_budget, max_ctx);
  if (dtype == DT_F16) {
    if (rpw == 1) FIER_STEP_RPW(DT_F16, 1);
    if (rpw == 2) FIER_STEP_RPW(DT_F16, 2);
    if (rpw == 4) FIER_STEP_RPW(DT_F16, 4);
    FIER_STEP_RPW(DT_F16, 8);
  }
  if (rpw == 1) FIER_STEP_RPW(DT_BF16, 1);
  if (rpw == 2) FIER_STEP_RPW(DT_BF16, 2);
  if (rpw == 4) FIER_STEP_RPW(DT_BF16, 4);
  FIER_STEP_RPW(DT_BF16, 8);
#undef FIER_STEP_RPW
}

// Whether the step's second part is one launch (step_attend_kernel) for this shape.
bool step_two_kernel_form(int units, int n_rep, int max_budget, int max_ctx, bool with_index_list) {
  // Measured against the threshold kernel + selection-and-attention kernel (us per step, fp16, budget = 11 % of the
  // context unless noted): with 4 query heads per kv head, 8 units x 32k 25.8 / 28.5, 64 x 32k 57.0 / 62.0, 128 x 32k
  // 95.7 / 108.8, 32 x 128k (budget 4096) 65.7 / 71.5, and on grids that are not resident at once 64 x 128k 121.2 /
  // 118.0, 256 x 32k 194.2 / 191.9; with one query head per kv head on such grids 256 x 128k 391 / 425, 2048 x 4k
  // 194 / 215, 1024 x 32k 664 / 698, 512 x 32k 341 / 348, 1024 x 8k 214 / 206.
  //   On the ragged batch of 128 such units x 8k..64k (budget 11 % of each length), whose grid at full length is 1.5
  //   times the resident one: 107 / 117.  Hence: always with 1 or 2 query heads per kv head; with more, up to twice
  //   the resident grid.
  //   With the ascending index list as an output the one-launch form needs one more kernel, which reads the scores
  //   again (config 2 +4.3 us, 32 units x 128k +10), while the selection + attention kernel writes the list as it
  //   selects: 32 x 128k at 4 heads per kv head 73.4 / 68.5, the ragged batch 115.3 / 108.7, 8 x 32k 29.3 / 28.5, but
  //   config 2 37.5 / 41.2.  Hence: with the list and 3 or more heads per kv head, three kernels.
  if (n_rep <= 2) return true;
  if (with_index_list) return false;
  const int rpw = step_ranges_per_wg(units, n_rep, max_budget, max_ctx);
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  return (long)units * ((n_ranges + rpw - 1) / rpw) <= 2 * step_resident_wgs(n_rep);
}

hipError_t launch_step_emit_idx(const StepBuffers& sb, const int32_t* seq_lens, int extra, int max_budget, int32_t* idx,
                                int units, int n_rep, int n_kv_heads, int max_ctx, hipStream_t st) {
  // the same split into workgroups as the step's second kernel
  const int rpw = step_ranges_per_wg(units, n_rep, max_budget, max_ctx);
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const int n_wgs = (n_ranges + rpw - 1) / rpw;
  const dim3 grid(units, n_wgs);
#define FIER_EMIT(RPW)                                                                                              \
  step_emit_idx_kernel<RPW><<<grid, kStepThreads, 0, st>>>(sb.scores, seq_lens, extra, sb.ctl, sb.sel_cnt, n_wgs, \
                                                           max_budget, idx, n_kv_heads, max_ctx)
  if (rpw == 1) FIER_EMIT(1);
  else if (rpw == 2) FIER_EMIT(2);
  else if (rpw == 4) FIER_EMIT(4);
  else FIER_EMIT(8);
#undef FIER_EMIT
  return hipGetLastError();
}

}  // namespace fier
