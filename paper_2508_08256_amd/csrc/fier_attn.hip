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
#include "fier_attn_dev.h"
#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {
// Stand-alone attention (fier_sparse_attn: rows from an index list; fier_dense_attn: all rows).  grid (n_splits,
// units), block 256: a workgroup attends over rows_per_wg entries and stores one partial per query head; the unit's
// last workgroup merges the partials of the splits in use (arrival counter in the unit's control block).
// STREAM: the rows are loaded with the streaming hint (a gather with three or more query heads per kv head: its V
// rows only).
template <int DT, int NREP, bool STREAM>
__global__ __launch_bounds__(256) void attn_split_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                         const uint4* __restrict__ q, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ seq_lens, int extra,
                                                         int max_budget, int rows_per_wg, int n_splits,
                                                         float scale_log2e, float* __restrict__ po,
                                                         float* __restrict__ pm, float* __restrict__ pl,
                                                         UnitCtl* __restrict__ ctl, float* __restrict__ out,
                                                         int n_kv_heads, int max_ctx, int unit_major, KvLayout lay) {
  __shared__ float sh_o[NREP * kPartialFloats];
  __shared__ uint32_t flag;

  const int cn = threadIdx.x & 15;
  const int unit = unit_major ? blockIdx.x : blockIdx.y, split = unit_major ? blockIdx.y : blockIdx.x;
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
  if (n <= 0 && split == 0) {  // nothing to attend over: zeros
    for (int o = threadIdx.x; o < NREP * kD; o += 256) out[(size_t)unit * NREP * kD + o] = 0.f;
    return;
  }
  if (start >= n) return;
  const int end = n < start + rows_per_wg ? n : start + rows_per_wg;
  const int32_t* __restrict__ sel = idx ? idx + (size_t)unit * max_budget : nullptr;
  const KvRows kv = lay.rows_of(unit);
  // whole-cache attention over paged rows: the block numbers of this workgroup's rows wait in LDS
  __shared__ int32_t lblk[kAttnRowsDenseMax / 64];
  const bool window = !sel && kv.blocks != nullptr;
  if (window) {
    const int bi = (start >> kv.shift) + (int)threadIdx.x;
    if (threadIdx.x < kAttnRowsDenseMax / 64) lblk[threadIdx.x] = bi < lay.blocks_per_seq ? kv.blocks[bi] : 0;
    __syncthreads();
  }
  const int first_block = start >> kv.shift;
  // an index outside the cache places no row: the entry is skipped (it gets no weight)
  auto row_sel = [&](int j) {
    const int t = sel[j];
    return (t < 0 || t >= max_ctx) ? kNoRow : kv.row(t);
  };
  const size_t safe_row = kv.row(0);
  auto row_all = [&](int j) {
    return window ? (size_t)lblk[(j >> kv.shift) - first_block] * kv.block_stride + kv.base + (size_t)(j & kv.mask)
                  : kv.base + (size_t)j;
  };

  uint4 qr[NREP];
#pragma unroll
  for (int r = 0; r < NREP; ++r) qr[r] = q[((size_t)unit * NREP + r) * (kD / 8) + cn];

  AttnState<NREP> st;
  st.init();
  if constexpr (NREP >= 3) {
    const uint4* q_unit = q + (size_t)unit * NREP * (kD / 8);
    if (sel)
      attend_rows_mfma<DT, NREP, true, false, STREAM>(K, V, q_unit, row_sel, start, end, scale_log2e, st, sh_o, false,
                                                      safe_row);
    else
      attend_rows_mfma<DT, NREP, false, STREAM>(K, V, q_unit, row_all, start, end, scale_log2e, st, sh_o);
  } else {
    if (sel)
      attend_rows<DT, NREP, true, STREAM>(K, V, qr, row_sel, start, end, scale_log2e, st, safe_row);
    else
      attend_rows<DT, NREP, false, STREAM>(K, V, qr, row_all, start, end, scale_log2e, st);
  }
  store_partials<NREP, true>(st, sh_o, unit, n_splits, split, po, pm, pl);
  // the unit's last workgroup merges the partials of the splits in use
  const int used = (n + rows_per_wg - 1) / rows_per_wg;
  if (!last_arriver(&ctl[unit].arrive[0], (uint32_t)used, &flag)) return;
  merge_heads<NREP>(po, pm, pl, unit, n_splits, used, sh_o, out + (size_t)unit * NREP * kD);
  if (threadIdx.x == 0) ctl[unit].arrive[0] = 0;
}

// Third kernel of the fused decode step.  grid (ceil(n_ranges / RPW), units), block 256: the workgroup owns RPW
// consecutive 1024-token ranges of its unit (RPW is chosen by the host so that a workgroup has on the order of a
// hundred selected rows).  It re-reads their scores, applies the exact selection rule fixed by the threshold
// kernel, writes its part of the ascending index list, and attends over its selected rows straight from an LDS
// list -- the index list never has to be read back.  The unit's last workgroup merges the partials.
template <int DT, int NREP, int RPW>
__global__ __launch_bounds__(256) void select_attend_kernel(
    const float* __restrict__ scores, UnitCtl* __restrict__ ctl, const uint32_t* __restrict__ range_off,
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint4* __restrict__ q,
    const int32_t* __restrict__ seq_lens, int extra, int max_budget, float scale_log2e, float* __restrict__ po,
    float* __restrict__ pm, float* __restrict__ pl, int32_t* __restrict__ idx_out, float* __restrict__ out,
    float* __restrict__ kabsmax, const float* __restrict__ newmax, int n_ranges, int n_kv_heads, int max_ctx,
    int order, int wgs_per_unit, KvLayout lay) {
  __shared__ float sh_o[NREP * kPartialFloats > 4 * 130 ? NREP * kPartialFloats : 4 * 130];
  __shared__ uint16_t rows[kRangeTokens * RPW];  // selected tokens, relative to the workgroup's first token
  __shared__ uint32_t scan_tmp[4];
  __shared__ uint32_t flag;
  __shared__ int32_t lblk[RPW * kRangeTokens / 64];  // paged rows: block numbers of this workgroup's tokens

  const int tid = threadIdx.x;
  const int cn = tid & 15;
  // order: 0 = grid (workgroups, units); 1 = grid (units, workgroups); 2 = one-dimensional, groups of 8 units, a
  // group's workgroups together and unit % 8 fastest (see the launcher)
  int unit, wg;
  if (order == 2) {
    const int id = blockIdx.x;
    const int g = id / (8 * wgs_per_unit);
    const int rem = id - g * 8 * wgs_per_unit;
    wg = rem >> 3;
    unit = 8 * g + (rem & 7);
  } else {
    unit = order ? blockIdx.x : blockIdx.y;
    wg = order ? blockIdx.y : blockIdx.x;
  }
  const int b = unit / n_kv_heads;
  int n = seq_lens[b] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  const int tok0 = wg * RPW * kRangeTokens;
  if (tok0 >= n && wg != 0) return;
  FIER_PROF(20, unit == 0 && wg == 3)
  FIER_PROF_WG(5)
  const KvRows kv = lay.rows_of(unit);
  if (kv.blocks && tid < RPW * kRangeTokens / 64) {  // in flight during the selection; barriers follow
    const int bi = (tok0 >> kv.shift) + tid;
    lblk[tid] = bi < lay.blocks_per_seq ? kv.blocks[bi] : 0;
  }
  UnitCtl* __restrict__ c = &ctl[unit];
  const int tbin = c->tbin;
  const float R = c->R, hscale = c->scale;
  const uint32_t T = c->T;
  const int32_t idxT = c->idxT;
  const int n_slots = wgs_per_unit;

  // ---- exact selection inside this workgroup's ranges, in token order ---------------------------------------
  float4 v[RPW];
  uint32_t off[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    v[rr] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n) v[rr] = *reinterpret_cast<const float4*>(scores + (size_t)unit * max_ctx + i);
    const int r = wg * RPW + rr;
    off[rr] = r < n_ranges ? range_off[(size_t)unit * n_ranges + r] : 0;
  }
  // selection flags of the thread's 4 tokens in each range, and their count
  uint32_t selm[RPW], cnt[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    const float vv[4] = {v[rr].x, v[rr].y, v[rr].z, v[rr].w};
    selm[rr] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int bin = sel_bin(vv[j], R, hscale, kSelBins);
      const uint32_t key = score_key(vv[j]);
      const bool sel = i + j < n && (bin > tbin || (bin == tbin && (key > T || (key == T && i + j <= idxT))));
      selm[rr] |= sel ? 1u << j : 0u;
    }
    cnt[rr] = __builtin_popcount(selm[rr]);
  }
  // positions in token order: one workgroup scan serves two ranges (16 bits each: a range holds <= 1024 tokens)
  uint32_t n_sel_total = 0;
#pragma unroll
  for (int r2 = 0; r2 < RPW; r2 += 2) {
    const uint32_t packed = cnt[r2] | (r2 + 1 < RPW ? cnt[r2 + 1 < RPW ? r2 + 1 : r2] << 16 : 0u);
    uint32_t total;
    const uint32_t before = block_excl_scan_u32<4>(packed, scan_tmp, total);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int rr = r2 + h;
      if (rr < RPW) {
        const int i = tok0 + rr * kRangeTokens + 4 * tid;
        uint32_t pos = (before >> (16 * h)) & 0xffffu;
        const uint32_t n_sel = (total >> (16 * h)) & 0xffffu;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (selm[rr] >> j & 1u) {
            rows[n_sel_total + pos] = (uint16_t)(i + j - tok0);
            if (idx_out && off[rr] + pos < (uint32_t)max_budget)
              idx_out[(size_t)unit * max_budget + off[rr] + pos] = i + j;
            ++pos;
          }
        n_sel_total += n_sel;
      }
    }
  }
  __syncthreads();
  FIER_PROF(21, unit == 0 && wg == 3)

  // ---- attention over the selected rows of these ranges --------------------------------------------------------
  uint4 qr[NREP];
#pragma unroll
  for (int h = 0; h < NREP; ++h) qr[h] = q[((size_t)unit * NREP + h) * (kD / 8) + cn];
  AttnState<NREP> st;
  st.init();
  const int first_block = tok0 >> kv.shift;
  auto row_of = [&](int j) {
    const int t = tok0 + (int)rows[j];
    return kv.blocks ? (size_t)lblk[(t >> kv.shift) - first_block] * kv.block_stride + kv.base + (size_t)(t & kv.mask)
                     : kv.base + (size_t)t;
  };
  if constexpr (NREP >= 3)
    attend_rows_mfma<DT, NREP, false, false, true>(K, V, q + (size_t)unit * NREP * (kD / 8), row_of, 0, (int)n_sel_total,
                                                   scale_log2e, st,
                               sh_o);
  else
    attend_rows<DT, NREP>(K, V, qr, row_of, 0, (int)n_sel_total, scale_log2e, st);
  FIER_PROF(22, unit == 0 && wg == 3)
  store_partials<NREP, true>(st, sh_o, unit, n_slots, wg, po, pm, pl);
  FIER_PROF(23, unit == 0 && wg == 3)
  FIER_PROF_WG(6)

  const int n_wgs = (n + RPW * kRangeTokens - 1) / (RPW * kRangeTokens);  // workgroups of this unit in use
  if (!last_arriver(&c->arrive[2], n_wgs > 0 ? (uint32_t)n_wgs : 1u, &flag)) return;
  FIER_PROF(24, unit == 0)
  // ---- the unit's last workgroup merges the partials of all workgroups --------------------------------------
  merge_heads<NREP>(po, pm, pl, unit, n_slots, n_wgs, sh_o, out + (size_t)unit * NREP * kD);
  if (tid == 0) c->arrive[2] = 0;
  FIER_PROF(25, unit == 0)
  FIER_PROF_WG(7)
  // the step appended a row: fold the bound of its re-quantized group into the unit's per-channel bound
  if (extra && seq_lens[b] < max_ctx && tid < kD) {
    float* slot = kabsmax + (size_t)unit * kD + tid;
    const float a = newmax[(size_t)unit * kD + tid];
    if (a > *slot) *slot = a;
  }
}

template <int DT>
static hipError_t launch_attn_dt(KvLayout lay, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                                 const int32_t* count, const int32_t* seq_lens, int extra, int max_budget,
                                 int rows_per_wg, int n_splits, float sm_scale, float* po, float* pm, float* pl,
                                 UnitCtl* ctl, float* out, int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  // dispatch order as in the select + attend kernel, for gathers; whole-cache attention streams and gains nothing
  const int unit_major = idx != nullptr && (long)units * n_splits <= 2 * 256L * (n_rep >= 3 ? 4 : 7) ? 1 : 0;
  dim3 grid = unit_major ? dim3(units, n_splits) : dim3(n_splits, units);
  const float sl2 = sm_scale * 1.4426950408889634f;
  if (!idx && rows_per_wg > kAttnRowsDenseMax) return hipErrorInvalidValue;  // the kernel's block-number window
  // Whole-cache attention reads every row once: from 64 MB of rows on they are loaded with the streaming hint
  // (measured: 32 units x 32k 98-101 -> 90-91 us, 32 x 64k 186 -> 165-172, 32 x 128k at 4 heads per kv head 398-406 ->
  // 384; 8 units x 4k, which the caches hold, 15.5 -> 19.2 with it).
  const bool stream = idx == nullptr ? (long)units * max_ctx * (2 * kD * 2) >= (64L << 20)
                                     : (long)units * max_budget * (2 * kD * 2) >= (8L << 20);  // as in the fused step
#define FIER_ATTN_ARGS                                                                                             \
  (const uint4*)K, (const uint4*)V, (const uint4*)q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits, \
      sl2, po, pm, pl, ctl, out, n_kv_heads, max_ctx, unit_major, lay
#define FIER_ATTN_CASE(R)                                                                                          \
  case R:                                                                                                          \
    if (stream) attn_split_kernel<DT, R, true><<<grid, 256, 0, st>>>(FIER_ATTN_ARGS);                              \
    else attn_split_kernel<DT, R, false><<<grid, 256, 0, st>>>(FIER_ATTN_ARGS);                                    \
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
#undef FIER_ATTN_ARGS
  return hipGetLastError();
}

template <int DT, int RPW>
static hipError_t launch_select_attend_dt(KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                          const void* q, const int32_t* seq_lens, int extra, int max_budget,
                                          float sm_scale, int32_t* idx_out, float* out, float* kabsmax, int units,
                                          int n_kv_heads, int max_ctx, hipStream_t st) {
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const int n_wgs = (n_ranges + RPW - 1) / RPW;
  // Dispatch order.  Workgroups go round-robin to the 8 XCDs in the order of their linear index; when a unit's
  // workgroups all run on one XCD, its scores, offsets, partials and arrival counter stay in that XCD's L2.
  //   1: units fastest (a multiple of 8 units puts unit u on XCD u % 8), for grids of at most about two resident
  //      rounds (256 CUs x 4 workgroups of this kernel for 3+ query heads per kv head, x 7 otherwise):
  //      20.8 -> 19.6 us at config 2, 29.4 -> 26.5 us at config 3 against order 0;
  //   2: longer grids with a multiple of 8 units: groups of 8 units one after the other, inside a group the
  //      workgroups in range order and unit % 8 fastest -- the same XCD assignment, but a sequence's ranges stay
  //      together in time (the ragged 128-unit batch: 69.9 -> 62.9 us against order 0; order 1 there: 75.5 us);
  //   0: ranges fastest, otherwise.
  const int order = (long)units * n_wgs <= 2 * 256L * (n_rep >= 3 ? 4 : 7) ? 1 : (units % 8 == 0 ? 2 : 0);
  dim3 grid = order == 2 ? dim3((unsigned)units * (unsigned)n_wgs) : (order ? dim3(units, n_wgs) : dim3(n_wgs, units));
  const float sl2 = sm_scale * 1.4426950408889634f;
#define FIER_SA_CASE(R)                                                                                            \
  case R:                                                                                                          \
    select_attend_kernel<DT, R, RPW><<<grid, 256, 0, st>>>(                                                        \
        sb.scores, sb.ctl, sb.range_cnt, (const uint4*)K, (const uint4*)V, (const uint4*)q, seq_lens, extra,       \
        max_budget, sl2, sb.po, sb.pm, sb.pl, idx_out, out, kabsmax, sb.newmax, n_ranges, n_kv_heads, max_ctx,     \
        order, n_wgs, lay);                                                                                        \
    break;
  switch (n_rep) {
    FIER_SA_CASE(1)
    FIER_SA_CASE(2)
    FIER_SA_CASE(3)
    FIER_SA_CASE(4)
    FIER_SA_CASE(5)
    FIER_SA_CASE(6)
    FIER_SA_CASE(7)
    FIER_SA_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_SA_CASE
  return hipGetLastError();
}

// Ranges per workgroup (rows per 1024-token range = 1024 * budget / context): at least 96 selected rows per workgroup,
// and twice that -- up to 288 rows -- where the grid is far beyond what the chip holds at once (more than two rounds)
// or a unit has more than 64 workgroups (its merge then reads that many partials).  Measured (us per step; 32 query
// / 8 kv heads): batch 16 x 16k at 11 % 67.2 -> 61.1, batch 8 x 64k 110.8 -> 105.4, the ragged 16-sequence batch
// 63.7 -> 61.8 (this kernel), batch 1 x 128k at 11 % 48.3 -> 46.0 with twice the ranges; but batch 1 x 32k 28.0 ->
// 30.6, batch 2 x 32k (24 query heads) 32.2 -> 34.0, batch 4 x 32k 41.7 -> 42.5, and the 4 x 128k shape at B = 4096
// 26.8 -> 29.4 (this kernel) -- grids of about one round -- lose by it, as does halving (64 rows: 34.4).
int select_attend_ranges_per_wg(int units, int n_rep, int max_budget, int max_ctx) {
  const double per_range = 1024.0 * (double)max_budget / (double)max_ctx;
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const long capacity = 256L * (n_rep >= 3 ? 4 : 7);  // workgroups of this kernel resident at once
  int rpw = 1;
  while (rpw < 8 && per_range * rpw < 96.0) rpw *= 2;
  while (rpw < 8 && per_range * (2 * rpw) <= 288.0) {
    const long per_unit = (n_ranges + rpw - 1) / rpw;
    if (per_unit * units <= 2 * capacity && per_unit <= 64) break;
    rpw *= 2;
  }
  return rpw;
}

hipError_t launch_select_attend(int dtype, KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                const void* q, const int32_t* seq_lens, int extra, int max_budget, float sm_scale,
                                int32_t* idx_out, float* out, float* kabsmax, int units, int n_kv_heads, int max_ctx,
                                hipStream_t st) {
#define FIER_SA_RPW(DT, RPW)                                                                                        \
  return launch_select_attend_dt<DT, RPW>(lay, n_rep, sb, K, V, q, seq_lens, extra, max_budget, sm_scale, idx_out, out, \
                                          kabsmax, units, n_kv_heads, max_ctx, st)
  const int rpw = select_attend_ranges_per_wg(units, n_rep, max_budget, max_ctx);
  if (dtype == DT_F16) {
    if (rpw == 1) FIER_SA_RPW(DT_F16, 1);
    if (rpw == 2) FIER_SA_RPW(DT_F16, 2);
    if (rpw == 4) FIER_SA_RPW(DT_F16, 4);
    FIER_SA_RPW(DT_F16, 8);
  }
  if (rpw == 1) FIER_SA_RPW(DT_BF16, 1);
  if (rpw == 2) FIER_SA_RPW(DT_BF16, 2);
  if (rpw == 4) FIER_SA_RPW(DT_BF16, 4);
  FIER_SA_RPW(DT_BF16, 8);
#undef FIER_SA_RPW
}

hipError_t launch_attn(int dtype, KvLayout lay, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                       const int32_t* count, const int32_t* seq_lens, int extra, int max_budget, int rows_per_wg,
                       int n_splits, float sm_scale, float* po, float* pm, float* pl, UnitCtl* ctl, float* out,
                       int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  if (dtype == DT_F16)
    return launch_attn_dt<DT_F16>(lay, n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                                  sm_scale, po, pm, pl, ctl, out, units, n_kv_heads, max_ctx, st);
  return launch_attn_dt<DT_BF16>(lay, n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                                 sm_scale, po, pm, pl, ctl, out, units, n_kv_heads, max_ctx, st);
}

}  // namespace fier
