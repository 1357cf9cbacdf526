// Internal launch interface between the C-ABI layer (fier_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fier {

// ---- where the K / V rows live -----------------------------------------------------------------------------------------
// Contiguous caches hold row t of unit u at row u * max_ctx + t.  Paged caches (a block table, as serving stacks keep
// ragged batches) hold the rows in pools [n_blocks][n_kv_heads][block_tokens][D]; sequence b's logical block j is
// pool block table[b * blocks_per_seq + j].  block_tokens is a power of two >= 64, so the 64 tokens of a pair block,
// a quantization group and a page always lie inside one block.
struct KvRows {  // the rows of one unit
  const int32_t* blocks;  // the sequence's block list; nullptr: contiguous
  size_t base;            // contiguous: u * max_ctx; paged: head * block_tokens
  size_t block_stride;    // paged: rows per pool block = n_kv_heads * block_tokens
  int shift, mask;        // log2(block_tokens), block_tokens - 1
  __device__ __forceinline__ size_t row(int t) const {
    return blocks ? (size_t)blocks[t >> shift] * block_stride + base + (size_t)(t & mask) : base + (size_t)t;
  }
};
struct KvLayout {  // one cache; passed to the kernels by value
  const int32_t* table;  // [batch][blocks_per_seq]; nullptr: contiguous
  int blocks_per_seq, shift, n_kv_heads, max_ctx;
  __device__ __forceinline__ KvRows rows_of(int unit) const {
    KvRows r;
    if (table) {
      const int b = unit / n_kv_heads, h = unit - b * n_kv_heads;
      r.blocks = table + (size_t)b * blocks_per_seq;
      r.base = (size_t)h << shift;
      r.block_stride = (size_t)n_kv_heads << shift;
    } else {
      r.blocks = nullptr;
      r.base = (size_t)unit * max_ctx;
      r.block_stride = 0;
    }
    r.shift = shift;
    r.mask = (1 << shift) - 1;
    return r;
  }
};

constexpr int kAttnRowsSparse = 128;  // selected rows per workgroup of the split attention kernel
constexpr int kAttnRowsDenseMin = 512;   // rows per workgroup when attending over the whole cache: the launcher
constexpr int kAttnRowsDenseMax = 3200;  // picks a multiple of 128 in this range (see dense_rows_per_wg)

// ---- fused decode step -------------------------------------------------------------------------------
// Per layer: (1) append + score + score histogram, (2) exact threshold + attention over the selected rows + merge --
// (2) is one kernel for up to 2 query heads per kv head and, unless the index list is asked for, on grids of up to
// twice the workgroups resident at once; it is split into a threshold kernel and a selection + attention kernel otherwise.  Each unit's tokens are spread over many
// workgroups; the few serial steps (exact threshold among the candidates of the threshold bin, merge of the
// attention partials) are done by one workgroup of the unit, as a rule the one that arrives last at a device-scope
// counter ("last arriver").  fier_topk_ws reuses the threshold kernel.
constexpr int kSelBins = 512;          // equal-width score histogram bins over [-R, R] (few enough that the
                                       // per-workgroup histograms merge with ~100 device atomics each)
constexpr int kRangeTokens = 1024;     // tokens per range: the unit of work of the step's second kernel
constexpr int kClassifyTokens = 4096;  // tokens per stretch of a threshold-kernel workgroup
constexpr int kSegCand = 1024;         // candidate slots per workgroup of that kernel
constexpr int kSelCandMax = 4096;      // candidates per unit its exact selection handles in LDS
constexpr int kSubBins = 1024;         // second-level bins inside the threshold bin
constexpr int kSubCandMax = 512;       // members of the threshold sub-bin ranked pairwise

struct UnitCtl {        // one per unit at the head of the workspace
  uint32_t arrive[3];   // arrival counters: [0] stand-alone attention,
                        // [1] classification (step) / threshold kernel, [2] attention partials of the step (upper
                        // half: workgroups whose partial lacks their threshold-bin rows); zero between calls
  uint32_t topk_max;    // fier_topk_ws: bit pattern of the largest |score| of the unit; zero between calls
  int32_t tbin;         // bins above are selected, bins below are not (-1: everything, kSelBins: nothing)
  uint32_t above;       // tokens in bins above tbin
  int32_t budget;       // tokens to select = min(budget, length, max_budget), >= 0
  float R;              // scores lie in [-R, R]
  float scale;          // kSelBins / (2 R)
  uint32_t T;           // threshold key inside tbin
  int32_t idxT;         // among keys == T inside tbin, indices <= idxT are selected
  uint32_t pad;
  unsigned long long thr;  // the step's threshold as one word, T << 32 | idxT + 2, published by the unit's selector
                           // to its other workgroups; zero between calls
  uint32_t chk_cnt;     // checksums of the rows the step attended over (count, sum of token indices); only
  uint32_t chk_sum;     // accumulated on request (tests), never cleared by the library
};
static_assert(sizeof(UnitCtl) == 64, "UnitCtl is one 64-byte line");

struct StepBuffers {    // carved from the caller's workspace
  UnitCtl* ctl;         // [units]
  uint32_t* hist;       // [units][kSelBins]: filled by the score kernel, read and cleared by the step's second kernel
  uint32_t* range_cnt;  // [units][n_ranges] (fier_topk_ws): selected tokens per 1024-token range, then their scan
  unsigned long long* cand;  // [units][cand_pitch] candidates (key << 32 | token index)
  uint32_t* seg_cnt;    // [units][seg_pitch] candidates published by each workgroup
  uint32_t* sel_cnt;    // [units][seg_pitch] rows each workgroup of the step's second kernel selected (for the
                        // index-list kernel)
  float* scores;        // [units][max_ctx]
  float* newmax;        // [units][128]: |dequantized key| bound of the group re-quantized by this step's append
  float* po;            // attention partials, n_ranges + 1 slots per (unit, query head)
  float* pm;
  float* pl;
  size_t cand_pitch;    // candidate slots per unit
  int seg_pitch;        // workgroup entries per unit in seg_cnt and sel_cnt
};

hipError_t launch_quantize(int dtype, KvLayout lay, const void* K, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                           const int32_t* seq_lens, int units, int n_kv_heads, int max_ctx, int group_size,
                           hipStream_t st);

hipError_t launch_append(int dtype, KvLayout lay, void* K, void* V, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                         const int32_t* seq_lens, const void* k_new, const void* v_new, int units, int n_kv_heads,
                         int max_ctx, int group_size, hipStream_t st);

// With sb != nullptr the kernel also builds the per-unit score histogram (first kernel of the fused step); with
// k_new != nullptr as well it appends the new K/V rows first (extra must then be 1).
hipError_t launch_score(int dtype, KvLayout lay, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                        const void* q, const int32_t* seq_lens, int extra, float* scores, const StepBuffers* sb,
                        const int32_t* budgets, int max_budget, void* K, void* V, const void* k_new,
                        const void* v_new, int units, int n_kv_heads, int max_ctx, int group_size, hipStream_t st);

// The same selection by many workgroups per unit where a unit's scores do not fit one workgroup's registers.
hipError_t launch_topk_ws(const StepBuffers& sb, const float* scores, const int32_t* seq_lens, int extra,
                          const int32_t* budgets, int max_budget, int32_t* idx, int32_t* count, int units,
                          int n_kv_heads, int max_ctx, hipStream_t st);

hipError_t launch_threshold(const StepBuffers& sb, const int32_t* seq_lens, int extra, const int32_t* budgets,
                            int max_budget, int32_t* count_out, int units, int n_kv_heads, int max_ctx,
                            hipStream_t st);

hipError_t launch_select_attend(int dtype, KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                const void* q, const int32_t* seq_lens, int extra, int max_budget, float sm_scale,
                                int32_t* idx_out, float* out, float* kabsmax, int units, int n_kv_heads, int max_ctx,
                                hipStream_t st);

// Second kernel of the fused step: exact threshold, attention over the selected rows, merge.  count_out may be null.
// flags (tests): bit 0 = no workgroup picks up the threshold itself (the merger's fallback does all threshold-bin rows),
// bit 1 = accumulate the checksums of the attended rows in the control blocks.
hipError_t launch_step_attend(int dtype, KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                              const void* q, const int32_t* seq_lens, int extra, const int32_t* budgets, int max_budget,
                              float sm_scale, int32_t* count_out, float* out, float* kabsmax, int units, int n_kv_heads,
                              int max_ctx, int flags, hipStream_t st);
// The ascending index list of the selection that kernel made (an optional output of the step).
hipError_t launch_step_emit_idx(const StepBuffers& sb, const int32_t* seq_lens, int extra, int max_budget, int32_t* idx,
                                int units, int n_rep, int n_kv_heads, int max_ctx, hipStream_t st);
int step_ranges_per_wg(int units, int n_rep, int max_budget, int max_ctx);
bool step_two_kernel_form(int units, int n_rep, int max_budget, int max_ctx, bool with_index_list);

hipError_t launch_topk(const float* scores, const int32_t* seq_lens, int extra, const int32_t* budgets,
                       int max_budget, int32_t* idx, int32_t* count, int units, int n_kv_heads, int max_ctx,
                       hipStream_t st);

// idx == nullptr: attend over rows [0, seq_len + extra) (dense).  rows_per_wg rows of the selection per
// workgroup; partials (po, pm, pl) hold n_splits entries per (unit, query head).
hipError_t launch_attn(int dtype, KvLayout lay, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                       const int32_t* count, const int32_t* seq_lens, int extra, int max_budget, int rows_per_wg,
                       int n_splits, float sm_scale, float* po, float* pm, float* pl, UnitCtl* ctl, float* out, int units,
                       int n_kv_heads, int max_ctx, hipStream_t st);

// ---- page-level importance (comparison workload) -------------------------------------------------------------------
hipError_t launch_page_minmax(int dtype, KvLayout lay, const void* K, const int32_t* seq_lens, uint32_t* page_meta, int units,
                              int n_kv_heads, int max_ctx, int P, hipStream_t st);
hipError_t launch_page_append(int dtype, const void* k_new, const int32_t* seq_lens, uint32_t* page_meta, int units,
                              int n_kv_heads, int max_ctx, int P, hipStream_t st);
hipError_t launch_page_score(int dtype, int n_rep, const uint32_t* page_meta, const void* q, const int32_t* seq_lens,
                             int extra, int mode, float* out, int units, int n_kv_heads, int max_ctx, int P,
                             hipStream_t st);
hipError_t launch_page_mean(const float* scores, const int32_t* seq_lens, int extra, float* out, int units,
                            int n_kv_heads, int max_ctx, int P, hipStream_t st);
hipError_t launch_expand_pages(const int32_t* page_idx, const int32_t* page_count, int max_pages,
                               const int32_t* seq_lens, int extra, int P, int32_t* idx, int32_t* count,
                               int max_budget, int units, int n_kv_heads, int max_ctx, hipStream_t st);

}  // namespace fier
