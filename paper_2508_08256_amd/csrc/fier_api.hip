// C-ABI entry points of libfier (declared in include/fier.h): argument validation on the host,
// workspace carving, and kernel enqueue.  No allocation, no synchronisation, no global state.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <mutex>

#include "fier.h"
#include "fier_kernels.h"

namespace {

constexpr int kD = 128;
constexpr int kPair = 64;
constexpr size_t kAlign = 256;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_cfg(const fier_config* c) {
  if (!c) return FIER_EINVAL;
  if (c->batch <= 0 || c->n_kv_heads <= 0 || c->n_q_heads <= 0 || c->max_ctx <= 0) return FIER_EINVAL;
  if (c->kv_dtype != FIER_F16 && c->kv_dtype != FIER_BF16) return FIER_EINVAL;
  if (!(c->sm_scale == c->sm_scale)) return FIER_EINVAL;
  if (c->head_dim != kD) return FIER_EUNSUPPORTED;
  if (c->group_size != 32 && c->group_size != 64 && c->group_size != 128 && c->group_size != 256)
    return FIER_EUNSUPPORTED;
  if (c->n_q_heads % c->n_kv_heads != 0) return FIER_ESHAPE;
  if (c->n_q_heads / c->n_kv_heads > 8) return FIER_EUNSUPPORTED;
  if (c->max_ctx % kPair != 0 || c->max_ctx % c->group_size != 0 || c->max_ctx > (1 << 20)) return FIER_ESHAPE;
  if ((int64_t)c->batch * c->n_kv_heads > 65535) return FIER_ESHAPE;
  return FIER_OK;
}

// Block-table fields of a cache: absent (contiguous rows), or a power-of-two block size that holds whole pair
// blocks, quantization groups and pages and divides the row capacity.
int check_blocks(const fier_config* c, const fier_cache* k) {
  if (!k->block_table) return k->block_tokens == 0 ? FIER_OK : FIER_EINVAL;
  const int32_t bt = k->block_tokens;
  if (bt < kPair || (bt & (bt - 1)) != 0 || bt < c->group_size || c->max_ctx % bt != 0) return FIER_ESHAPE;
  if ((reinterpret_cast<uintptr_t>(k->block_table) & 3u) != 0) return FIER_EALIGN;
  return FIER_OK;
}

int check_cache(const fier_config* c, const fier_cache* k) {
  if (!k || !k->k || !k->v || !k->kbits || !k->kmeta || !k->kabsmax || !k->seq_lens) return FIER_EINVAL;
  if (misaligned(k->k) || misaligned(k->v) || misaligned(k->kbits) || misaligned(k->kmeta) ||
      misaligned(k->kabsmax))
    return FIER_EALIGN;
  return check_blocks(c, k);
}

// Where the K / V rows of the cache live (contiguous per unit, or in pool blocks through the block table).
fier::KvLayout layout_of(const fier_config* c, const fier_cache* k) {
  fier::KvLayout lay;
  lay.table = k->block_table;
  lay.n_kv_heads = c->n_kv_heads;
  lay.max_ctx = c->max_ctx;
  lay.shift = 0;
  lay.blocks_per_seq = 0;
  if (k->block_table) {
    while ((1 << lay.shift) < k->block_tokens) ++lay.shift;
    lay.blocks_per_seq = c->max_ctx / k->block_tokens;
  }
  return lay;
}

inline int units_of(const fier_config* c) { return c->batch * c->n_kv_heads; }
inline int n_rep_of(const fier_config* c) { return c->n_q_heads / c->n_kv_heads; }
inline int splits_for(int max_budget) { return (max_budget + fier::kAttnRowsSparse - 1) / fier::kAttnRowsSparse; }

// Rows per workgroup of whole-cache attention: about 640 workgroups in all (measured: the fewer and longer the
// workgroups the better, down to two or three per CU; config 2: 117 us at 512 rows, 99 us at 2304), a multiple of
// 128 that is not a power of two (such strides between the workgroups' streams collide in the memory channels).
inline int dense_rows_per_wg(const fier_config* c) {
  const long total = (long)units_of(c) * c->max_ctx;
  long rows = (total / 640 + 127) / 128 * 128;
  rows = rows < fier::kAttnRowsDenseMin ? fier::kAttnRowsDenseMin : rows;
  rows = rows > fier::kAttnRowsDenseMax - 128 ? fier::kAttnRowsDenseMax - 128 : rows;
  if ((rows & (rows - 1)) == 0) rows += 128;
  return (int)rows;
}

inline int ranges_of(const fier_config* c) { return (c->max_ctx + fier::kRangeTokens - 1) / fier::kRangeTokens; }

struct Workspace {
  fier::StepBuffers sb;  // fused step: control blocks, histograms, candidates, scores, partials
  float* po;             // stand-alone attention partials (split kernel + merge kernel)
  float* pm;
  float* pl;
  int32_t* idx;
  int32_t* count;
  size_t zero_bytes;  // the leading part that must be zero before the first call (control blocks, histograms)
  size_t bytes;
};

// Carve the workspace for selections of up to max_budget rows per unit.  base may be null (sizing only).
// The control blocks and histograms come first: they are the part that must be zero before the first call.
Workspace carve(const fier_config* c, int32_t max_budget, void* base) {
  const size_t units = (size_t)units_of(c), heads = units * (size_t)n_rep_of(c);
  const size_t splits = (size_t)splits_for(max_budget), ranges = (size_t)ranges_of(c);
  char* p = static_cast<char*>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* r = p + off;
    off += align_up(bytes);
    return r;
  };
  Workspace w;
  const size_t chunks = ((size_t)c->max_ctx + fier::kClassifyTokens - 1) / fier::kClassifyTokens;
  // candidate slots and workgroup entries per unit: enough for the step's second kernel (a quarter of the tokens of
  // up to n_ranges workgroups, rounded up to whole workgroups of 8 ranges) and for fier_topk_ws's threshold kernel
  const size_t cand_pitch = std::max(chunks * fier::kSegCand, (ranges + 8) * (size_t)(fier::kRangeTokens / 4));
  const size_t seg_pitch = std::max(chunks, ranges);
  w.sb.cand_pitch = cand_pitch;
  w.sb.seg_pitch = (int)seg_pitch;
  w.sb.ctl = reinterpret_cast<fier::UnitCtl*>(take(units * sizeof(fier::UnitCtl)));
  w.sb.hist = reinterpret_cast<uint32_t*>(take(units * fier::kSelBins * sizeof(uint32_t)));
  w.zero_bytes = off;
  w.sb.range_cnt = reinterpret_cast<uint32_t*>(take(units * ranges * sizeof(uint32_t)));
  w.sb.cand = reinterpret_cast<unsigned long long*>(take(units * cand_pitch * sizeof(unsigned long long)));
  w.sb.seg_cnt = reinterpret_cast<uint32_t*>(take(units * seg_pitch * sizeof(uint32_t)));
  w.sb.sel_cnt = reinterpret_cast<uint32_t*>(take(units * seg_pitch * sizeof(uint32_t)));
  w.sb.scores = reinterpret_cast<float*>(take(units * (size_t)c->max_ctx * sizeof(float)));
  w.sb.newmax = reinterpret_cast<float*>(take(units * kD * sizeof(float)));
  w.sb.po = reinterpret_cast<float*>(take(heads * (ranges + 1) * kD * sizeof(float)));
  w.sb.pm = reinterpret_cast<float*>(take(heads * (ranges + 1) * sizeof(float)));
  w.sb.pl = reinterpret_cast<float*>(take(heads * (ranges + 1) * sizeof(float)));
  w.po = reinterpret_cast<float*>(take(heads * splits * kD * sizeof(float)));
  w.pm = reinterpret_cast<float*>(take(heads * splits * sizeof(float)));
  w.pl = reinterpret_cast<float*>(take(heads * splits * sizeof(float)));
  w.idx = reinterpret_cast<int32_t*>(take(units * (size_t)max_budget * sizeof(int32_t)));
  w.count = reinterpret_cast<int32_t*>(take(units * sizeof(int32_t)));
  w.bytes = off;
  return w;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? FIER_OK : FIER_EHIP; }

// The caller's workspace against what the call is going to carve from it.
inline int check_workspace(const void* ws, size_t have, size_t need) {
  if (!ws || have < need) return FIER_EWORKSPACE;
  if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return FIER_EALIGN;
  return FIER_OK;
}

}  // namespace

extern "C" {

const char* fier_status_string(int status) {
  switch (status) {
    case FIER_OK: return "ok";
    case FIER_EINVAL: return "invalid argument";
    case FIER_ESHAPE: return "unsupported shape";
    case FIER_EALIGN: return "device pointer not 16-byte aligned";
    case FIER_EWORKSPACE: return "workspace missing or too small";
    case FIER_EUNSUPPORTED: return "unsupported configuration";
    case FIER_EHIP: return "kernel launch failed";
    default: return "unknown status";
  }
}

int fier_check_config(const fier_config* cfg) { return check_cfg(cfg); }

size_t fier_packed_bits_bytes(const fier_config* cfg) {
  if (check_cfg(cfg) != FIER_OK) return 0;
  return (size_t)units_of(cfg) * (size_t)cfg->max_ctx * 4 * sizeof(uint32_t);
}

size_t fier_packed_meta_bytes(const fier_config* cfg) {
  if (check_cfg(cfg) != FIER_OK) return 0;
  return (size_t)units_of(cfg) * (size_t)(cfg->max_ctx / cfg->group_size) * kD * sizeof(uint32_t);
}

size_t fier_workspace_bytes(const fier_config* cfg, int32_t max_budget) {
  if (check_cfg(cfg) != FIER_OK || max_budget < 1) return 0;
  if (max_budget > cfg->max_ctx) max_budget = cfg->max_ctx;
  return carve(cfg, max_budget, nullptr).bytes;
}

size_t fier_workspace_scores_offset(const fier_config* cfg, int32_t max_budget) {
  if (check_cfg(cfg) != FIER_OK || max_budget < 1) return 0;
  if (max_budget > cfg->max_ctx) max_budget = cfg->max_ctx;
  char* const base = reinterpret_cast<char*>(kAlign);  // any aligned address: only the distance matters
  const Workspace w = carve(cfg, max_budget, base);
  return static_cast<size_t>(reinterpret_cast<char*>(w.sb.scores) - base);
}

int fier_decode_step_kernels(const fier_config* cfg, int32_t max_budget, int32_t with_index_list) {
  if (check_cfg(cfg) != FIER_OK || max_budget < 1) return 0;
  if (max_budget > cfg->max_ctx) max_budget = cfg->max_ctx;
  return fier::step_two_kernel_form(units_of(cfg), n_rep_of(cfg), max_budget, cfg->max_ctx, with_index_list != 0) ? 2 : 3;
}

int fier_quantize_keys(const fier_config* cfg, const fier_cache* cache, void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  st = check_cache(cfg, cache);
  if (st != FIER_OK) return st;
  return hip_status(fier::launch_quantize(cfg->kv_dtype, layout_of(cfg, cache), cache->k, cache->kbits, cache->kmeta, cache->kabsmax,
                                          cache->seq_lens, units_of(cfg), cfg->n_kv_heads, cfg->max_ctx,
                                          cfg->group_size, (hipStream_t)stream));
}

int fier_append_key(const fier_config* cfg, const fier_cache* cache, const void* k_new, const void* v_new,
                    void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  st = check_cache(cfg, cache);
  if (st != FIER_OK) return st;
  if (!k_new || !v_new) return FIER_EINVAL;
  if (misaligned(k_new) || misaligned(v_new)) return FIER_EALIGN;
  return hip_status(fier::launch_append(cfg->kv_dtype, layout_of(cfg, cache), cache->k, cache->v, cache->kbits, cache->kmeta,
                                        cache->kabsmax, cache->seq_lens, k_new, v_new, units_of(cfg),
                                        cfg->n_kv_heads, cfg->max_ctx, cfg->group_size, (hipStream_t)stream));
}

int fier_score(const fier_config* cfg, const fier_cache* cache, const void* q, int32_t extra_tokens, float* scores,
               void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  st = check_cache(cfg, cache);
  if (st != FIER_OK) return st;
  if (!q || !scores || extra_tokens < 0 || extra_tokens > 1) return FIER_EINVAL;
  if (misaligned(q) || misaligned(scores)) return FIER_EALIGN;
  return hip_status(fier::launch_score(cfg->kv_dtype, layout_of(cfg, cache), n_rep_of(cfg), cache->kbits, cache->kmeta, cache->kabsmax, q,
                                       cache->seq_lens, extra_tokens, scores, nullptr, nullptr, 0, nullptr, nullptr,
                                       nullptr, nullptr, units_of(cfg), cfg->n_kv_heads, cfg->max_ctx,
                                       cfg->group_size, (hipStream_t)stream));
}

int fier_topk(const fier_config* cfg, const float* scores, const int32_t* seq_lens, int32_t extra_tokens,
              const int32_t* budgets, int32_t max_budget, int32_t* idx, int32_t* count, void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  if (!scores || !seq_lens || !budgets || !idx || !count) return FIER_EINVAL;
  if (extra_tokens < 0 || extra_tokens > 1 || max_budget < 1) return FIER_EINVAL;
  if (misaligned(scores) || misaligned(idx)) return FIER_EALIGN;
  return hip_status(fier::launch_topk(scores, seq_lens, extra_tokens, budgets, max_budget, idx, count, units_of(cfg),
                                      cfg->n_kv_heads, cfg->max_ctx, (hipStream_t)stream));
}

int fier_topk_ws(const fier_config* cfg, const float* scores, const int32_t* seq_lens, int32_t extra_tokens,
                 const int32_t* budgets, int32_t max_budget, int32_t* idx, int32_t* count, void* workspace,
                 size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  if (!scores || !seq_lens || !budgets || !idx || !count) return FIER_EINVAL;
  if (extra_tokens < 0 || extra_tokens > 1 || max_budget < 1) return FIER_EINVAL;
  if (misaligned(scores) || misaligned(idx)) return FIER_EALIGN;
  if (max_budget > cfg->max_ctx) max_budget = cfg->max_ctx;
  st = check_workspace(workspace, workspace_bytes, carve(cfg, max_budget, nullptr).bytes);
  if (st != FIER_OK) return st;
  Workspace w = carve(cfg, max_budget, workspace);
  return hip_status(fier::launch_topk_ws(w.sb, scores, seq_lens, extra_tokens, budgets, max_budget, idx, count,
                                         units_of(cfg), cfg->n_kv_heads, cfg->max_ctx, (hipStream_t)stream));
}

int fier_sparse_attn(const fier_config* cfg, const fier_cache* cache, const void* q, const int32_t* idx,
                     const int32_t* count, int32_t max_budget, float* out, void* workspace, size_t workspace_bytes,
                     void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  st = check_cache(cfg, cache);
  if (st != FIER_OK) return st;
  if (!q || !idx || !count || !out || max_budget < 1) return FIER_EINVAL;
  if (misaligned(q) || misaligned(idx) || misaligned(out)) return FIER_EALIGN;
  if (max_budget > cfg->max_ctx) return FIER_EINVAL;
  st = check_workspace(workspace, workspace_bytes, carve(cfg, max_budget, nullptr).bytes);
  if (st != FIER_OK) return st;
  Workspace w = carve(cfg, max_budget, workspace);
  return hip_status(fier::launch_attn(cfg->kv_dtype, layout_of(cfg, cache), n_rep_of(cfg), cache->k, cache->v, q, idx, count,
                                      cache->seq_lens, 0, max_budget, fier::kAttnRowsSparse, splits_for(max_budget),
                                      cfg->sm_scale, w.po, w.pm, w.pl, w.sb.ctl, out, units_of(cfg), cfg->n_kv_heads,
                                      cfg->max_ctx, (hipStream_t)stream));
}

int fier_dense_attn(const fier_config* cfg, const fier_cache* cache, const void* q, int32_t extra_tokens, float* out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  st = check_cache(cfg, cache);
  if (st != FIER_OK) return st;
  if (!q || !out || extra_tokens < 0 || extra_tokens > 1) return FIER_EINVAL;
  if (misaligned(q) || misaligned(out)) return FIER_EALIGN;
  st = check_workspace(workspace, workspace_bytes, carve(cfg, cfg->max_ctx, nullptr).bytes);
  if (st != FIER_OK) return st;
  Workspace w = carve(cfg, cfg->max_ctx, workspace);
  const int rows_per_wg = dense_rows_per_wg(cfg);
  const int n_splits = (cfg->max_ctx + rows_per_wg - 1) / rows_per_wg;
  return hip_status(fier::launch_attn(cfg->kv_dtype, layout_of(cfg, cache), n_rep_of(cfg), cache->k, cache->v, q, nullptr, nullptr,
                                      cache->seq_lens, extra_tokens, cfg->max_ctx, rows_per_wg, n_splits,
                                      cfg->sm_scale, w.po, w.pm, w.pl, w.sb.ctl, out, units_of(cfg), cfg->n_kv_heads,
                                      cfg->max_ctx, (hipStream_t)stream));
}

static int decode_step_impl(const fier_config* cfg, const fier_cache* layers, int32_t n_layers,
                            const uint8_t* dense_layers, const void* q, const void* k_new, const void* v_new,
                            const int32_t* budgets, int32_t max_budget, float* out, int32_t* idx_out,
                            int32_t* count_out, void* workspace, size_t workspace_bytes, int32_t phase,
                            void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  if (!layers || n_layers < 1 || !q || !budgets || !out || max_budget < 1) return FIER_EINVAL;
  if ((k_new == nullptr) != (v_new == nullptr)) return FIER_EINVAL;
  if ((idx_out == nullptr) != (count_out == nullptr)) return FIER_EINVAL;
  // phase -1: validate only; 0: the whole step; 1, 2, 3: one kernel; 2 + 16 f, 3 + 16 f: kernels 2, 3 of the
  // two-kernel form with test flags f; 2 + 64, 3 + 64: kernels 2, 3 of the three-kernel form
  const bool phase_ok = (phase >= -1 && phase <= 3) ||
                        (phase > 3 && ((phase & 15) == 2 || (phase & 15) == 3) && (phase >> 4) <= 4);
  if (max_budget > cfg->max_ctx || !phase_ok) return FIER_EINVAL;
  if (misaligned(q) || misaligned(out) || misaligned(k_new) || misaligned(v_new) || misaligned(idx_out))
    return FIER_EALIGN;
  for (int l = 0; l < n_layers; ++l) {
    st = check_cache(cfg, &layers[l]);
    if (st != FIER_OK) return st;
  }
  // a layer that runs whole-cache attention carves the workspace for selections of max_ctx rows
  bool any_dense = false;
  for (int l = 0; dense_layers && l < n_layers; ++l) any_dense = any_dense || dense_layers[l] != 0;
  st = check_workspace(workspace, workspace_bytes, carve(cfg, any_dense ? cfg->max_ctx : max_budget, nullptr).bytes);
  if (st != FIER_OK) return st;
  if (phase < 0) return FIER_OK;
  const int units = units_of(cfg), n_rep = n_rep_of(cfg);
  const int extra = k_new ? 1 : 0;
  const size_t esz = 2;
  hipStream_t s = (hipStream_t)stream;
  Workspace w = carve(cfg, max_budget, workspace);
  for (int l = 0; l < n_layers; ++l) {
    const fier_cache* c = &layers[l];
    const char* ql = static_cast<const char*>(q) + (size_t)l * cfg->batch * cfg->n_q_heads * kD * esz;
    float* outl = out + (size_t)l * cfg->batch * cfg->n_q_heads * kD;
    int32_t* idxl = idx_out ? idx_out + (size_t)l * units * max_budget : nullptr;
    int32_t* cntl = count_out ? count_out + (size_t)l * units : nullptr;
    hipError_t e;
    const fier::KvLayout lay = layout_of(cfg, c);
    const char* kn = extra ? static_cast<const char*>(k_new) + (size_t)l * units * kD * esz : nullptr;
    const char* vn = extra ? static_cast<const char*>(v_new) + (size_t)l * units * kD * esz : nullptr;
    if (dense_layers && dense_layers[l]) {
      // full attention for this layer: append (the packed cache stays up to date), then attend over every row
      if (extra) {
        e = fier::launch_append(cfg->kv_dtype, lay, c->k, c->v, c->kbits, c->kmeta, c->kabsmax, c->seq_lens, kn, vn, units,
                                cfg->n_kv_heads, cfg->max_ctx, cfg->group_size, s);
        if (e != hipSuccess) return FIER_EHIP;
      }
      Workspace wd = carve(cfg, cfg->max_ctx, workspace);
      const int rows_per_wg = dense_rows_per_wg(cfg);
      const int n_splits = (cfg->max_ctx + rows_per_wg - 1) / rows_per_wg;
      e = fier::launch_attn(cfg->kv_dtype, lay, n_rep, c->k, c->v, ql, nullptr, nullptr, c->seq_lens, extra, cfg->max_ctx,
                            rows_per_wg, n_splits, cfg->sm_scale, wd.po, wd.pm, wd.pl, wd.sb.ctl, outl, units,
                            cfg->n_kv_heads, cfg->max_ctx, s);
      if (e != hipSuccess) return FIER_EHIP;
      continue;
    }
    if (phase == 0 || phase == 1) {
      e = fier::launch_score(cfg->kv_dtype, lay, n_rep, c->kbits, c->kmeta, c->kabsmax, ql, c->seq_lens, extra,
                             w.sb.scores, &w.sb, budgets, max_budget, c->k, c->v, kn, vn, units, cfg->n_kv_heads,
                             cfg->max_ctx, cfg->group_size, s);
      if (e != hipSuccess) return FIER_EHIP;
    }
    // After scoring: one launch (exact threshold + attention + merge, then the index list if asked for) wherever
    // that measured faster; grouped-query shapes take the threshold kernel and the selection + attention kernel,
    // whose workgroups never wait for each other, on grids far beyond the resident one and whenever the index list
    // is asked for (that form writes it while it selects).
    const bool two_kernels =
        phase > 3 ? (phase >> 4) <= 3
                  : fier::step_two_kernel_form(units, n_rep, max_budget, cfg->max_ctx, idx_out != nullptr);
    if (two_kernels) {
      if (phase == 0 || (phase & 15) == 2) {
        e = fier::launch_step_attend(cfg->kv_dtype, lay, n_rep, w.sb, c->k, c->v, ql, c->seq_lens, extra, budgets,
                                     max_budget, cfg->sm_scale, cntl, outl, c->kabsmax, units, cfg->n_kv_heads,
                                     cfg->max_ctx, phase >> 4, s);
        if (e != hipSuccess) return FIER_EHIP;
      }
      if ((phase == 0 || (phase & 15) == 3) && idxl) {
        e = fier::launch_step_emit_idx(w.sb, c->seq_lens, extra, max_budget, idxl, units, n_rep, cfg->n_kv_heads,
                                         cfg->max_ctx, s);
        if (e != hipSuccess) return FIER_EHIP;
      }
    } else {
      if (phase == 0 || (phase & 15) == 2) {
        e = fier::launch_threshold(w.sb, c->seq_lens, extra, budgets, max_budget, cntl, units, cfg->n_kv_heads,
                                   cfg->max_ctx, s);
        if (e != hipSuccess) return FIER_EHIP;
      }
      if (phase == 0 || (phase & 15) == 3) {
        e = fier::launch_select_attend(cfg->kv_dtype, lay, n_rep, w.sb, c->k, c->v, ql, c->seq_lens, extra, max_budget,
                                       cfg->sm_scale, idxl, outl, c->kabsmax, units, cfg->n_kv_heads, cfg->max_ctx, s);
        if (e != hipSuccess) return FIER_EHIP;
      }
    }
  }
  return FIER_OK;
}

int fier_decode_step(const fier_config* cfg, const fier_cache* layers, int32_t n_layers, const void* q,
                     const void* k_new, const void* v_new, const int32_t* budgets, int32_t max_budget, float* out,
                     int32_t* idx_out, int32_t* count_out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_step_impl(cfg, layers, n_layers, nullptr, q, k_new, v_new, budgets, max_budget, out, idx_out, count_out,
                          workspace, workspace_bytes, 0, stream);
}

int fier_decode_step_mixed(const fier_config* cfg, const fier_cache* layers, int32_t n_layers,
                           const uint8_t* dense_layers, const void* q, const void* k_new, const void* v_new,
                           const int32_t* budgets, int32_t max_budget, float* out, int32_t* idx_out,
                           int32_t* count_out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_step_impl(cfg, layers, n_layers, dense_layers, q, k_new, v_new, budgets, max_budget, out, idx_out,
                          count_out, workspace, workspace_bytes, 0, stream);
}

int fier_decode_step_phase(const fier_config* cfg, const fier_cache* layers, int32_t n_layers, const void* q,
                           const void* k_new, const void* v_new, const int32_t* budgets, int32_t max_budget,
                           float* out, int32_t* idx_out, int32_t* count_out, void* workspace,
                           size_t workspace_bytes, int32_t phase, void* stream) {
  if (phase < 1) return FIER_EINVAL;
  return decode_step_impl(cfg, layers, n_layers, nullptr, q, k_new, v_new, budgets, max_budget, out, idx_out, count_out,
                          workspace, workspace_bytes, phase, stream);
}

// ---- the step on library-owned scratch ------------------------------------------------------------------------------
// For callers that cannot allocate.  The workspace is a fixed array in the library's device image: every GPU the
// library runs on holds one copy at its own address until the process ends.  In host code the array's name is only
// a handle: the address kernels can use comes from hipGetSymbolAddress, asked once per device with that device current.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)48 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

__global__ void zero_words_kernel(uint32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Device address of the current device's copy of `scratch` (resolved on the first call on that device).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FIER_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FIER_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FIER_OK;
}
}  // namespace

int fier_decode_step_static(const fier_config* cfg, const fier_cache* layers, int32_t n_layers, const void* q,
                            const void* k_new, const void* v_new, const int32_t* budgets, int32_t max_budget,
                            float* out, int32_t* idx_out, int32_t* count_out, void* stream) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  if (max_budget < 1 || max_budget > cfg->max_ctx) return FIER_EINVAL;
  const Workspace need = carve(cfg, max_budget, nullptr);
  if (need.bytes > kStaticScratchBytes) return FIER_EWORKSPACE;  // beyond what the library holds
  // everything else is checked before the scratch is touched, so that an error leaves nothing enqueued
  st = decode_step_impl(cfg, layers, n_layers, nullptr, q, k_new, v_new, budgets, max_budget, out, idx_out, count_out,
                        reinterpret_cast<void*>(kAlign), kStaticScratchBytes, -1, stream);
  if (st != FIER_OK) return st;
  void* ptr = nullptr;
  st = static_scratch(&ptr);
  if (st != FIER_OK) return st;
  // The array keeps what the last call left, possibly laid out for another shape: the part that has to start at
  // zero is cleared by a kernel on the caller's stream (a fill kernel, not a memset node: callers may be capturing).
  const size_t words = need.zero_bytes / sizeof(uint32_t);
  zero_words_kernel<<<(unsigned)((words + 1023) / 1024 < 256 ? (words + 1023) / 1024 : 256), 256, 0,
                      (hipStream_t)stream>>>(static_cast<uint32_t*>(ptr), words);
  if (hipGetLastError() != hipSuccess) return FIER_EHIP;
  return decode_step_impl(cfg, layers, n_layers, nullptr, q, k_new, v_new, budgets, max_budget, out, idx_out, count_out,
                          ptr, kStaticScratchBytes, 0, stream);
}

// ---- page-level importance ------------------------------------------------------------------------------------------
static int check_page(const fier_config* cfg, int32_t page_tokens) {
  int st = check_cfg(cfg);
  if (st != FIER_OK) return st;
  if (page_tokens != 8 && page_tokens != 16 && page_tokens != 32) return FIER_EUNSUPPORTED;
  return FIER_OK;  // max_ctx is a multiple of 64, hence of the page size
}

size_t fier_page_meta_bytes(const fier_config* cfg, int32_t page_tokens) {
  if (check_page(cfg, page_tokens) != FIER_OK) return 0;
  return (size_t)units_of(cfg) * (size_t)(cfg->max_ctx / page_tokens) * kD * sizeof(uint32_t);
}

int fier_page_minmax(const fier_config* cfg, const fier_cache* cache, int32_t page_tokens, uint32_t* page_meta,
                     void* stream) {
  int st = check_page(cfg, page_tokens);
  if (st != FIER_OK) return st;
  if (!cache || !cache->k || !cache->seq_lens || !page_meta) return FIER_EINVAL;
  if (misaligned(cache->k) || misaligned(page_meta)) return FIER_EALIGN;
  st = check_blocks(cfg, cache);
  if (st != FIER_OK) return st;
  return hip_status(fier::launch_page_minmax(cfg->kv_dtype, layout_of(cfg, cache), cache->k, cache->seq_lens, page_meta, units_of(cfg),
                                             cfg->n_kv_heads, cfg->max_ctx, page_tokens, (hipStream_t)stream));
}

int fier_page_append(const fier_config* cfg, const int32_t* seq_lens, int32_t page_tokens, const void* k_new,
                     uint32_t* page_meta, void* stream) {
  int st = check_page(cfg, page_tokens);
  if (st != FIER_OK) return st;
  if (!seq_lens || !k_new || !page_meta) return FIER_EINVAL;
  if (misaligned(k_new) || misaligned(page_meta)) return FIER_EALIGN;
  return hip_status(fier::launch_page_append(cfg->kv_dtype, k_new, seq_lens, page_meta, units_of(cfg),
                                             cfg->n_kv_heads, cfg->max_ctx, page_tokens, (hipStream_t)stream));
}

int fier_page_score(const fier_config* cfg, const uint32_t* page_meta, int32_t page_tokens, const int32_t* seq_lens,
                    int32_t extra_tokens, const void* q, int32_t mode, float* page_scores, void* stream) {
  int st = check_page(cfg, page_tokens);
  if (st != FIER_OK) return st;
  if (!page_meta || !seq_lens || !q || !page_scores || extra_tokens < 0 || extra_tokens > 1 || mode < 0 || mode > 1)
    return FIER_EINVAL;
  if (misaligned(page_meta) || misaligned(q) || misaligned(page_scores)) return FIER_EALIGN;
  return hip_status(fier::launch_page_score(cfg->kv_dtype, n_rep_of(cfg), page_meta, q, seq_lens, extra_tokens, mode,
                                            page_scores, units_of(cfg), cfg->n_kv_heads, cfg->max_ctx, page_tokens,
                                            (hipStream_t)stream));
}

int fier_page_mean_score(const fier_config* cfg, const float* scores, const int32_t* seq_lens, int32_t extra_tokens,
                         int32_t page_tokens, float* page_scores, void* stream) {
  int st = check_page(cfg, page_tokens);
  if (st != FIER_OK) return st;
  if (!scores || !seq_lens || !page_scores || extra_tokens < 0 || extra_tokens > 1) return FIER_EINVAL;
  if (misaligned(scores) || misaligned(page_scores)) return FIER_EALIGN;
  return hip_status(fier::launch_page_mean(scores, seq_lens, extra_tokens, page_scores, units_of(cfg),
                                           cfg->n_kv_heads, cfg->max_ctx, page_tokens, (hipStream_t)stream));
}

int fier_expand_pages(const fier_config* cfg, const int32_t* page_idx, const int32_t* page_count, int32_t max_pages,
                      const int32_t* seq_lens, int32_t extra_tokens, int32_t page_tokens, int32_t* idx,
                      int32_t* count, int32_t max_budget, void* stream) {
  int st = check_page(cfg, page_tokens);
  if (st != FIER_OK) return st;
  if (!page_idx || !page_count || !seq_lens || !idx || !count || max_pages <= 0 || max_budget <= 0 ||
      extra_tokens < 0 || extra_tokens > 1)
    return FIER_EINVAL;
  return hip_status(fier::launch_expand_pages(page_idx, page_count, max_pages, seq_lens, extra_tokens, page_tokens,
                                              idx, count, max_budget, units_of(cfg), cfg->n_kv_heads, cfg->max_ctx,
                                              (hipStream_t)stream));
}

void fier_unpack_bits(const fier_config* cfg, const uint32_t* kbits_host, uint8_t* bits_host) {
  if (check_cfg(cfg) != FIER_OK || !kbits_host || !bits_host) return;
  const size_t n_tok = (size_t)units_of(cfg) * (size_t)cfg->max_ctx;
  for (size_t t = 0; t < n_tok; ++t)
    for (int d = 0; d < 4; ++d) {
      const uint32_t w = kbits_host[t * 4 + d];
      for (int i = 0; i < 32; ++i) {
        const int c = 64 * (d & 1) + 2 * i + (d >> 1);
        bits_host[t * kD + c] = (uint8_t)((w >> i) & 1u);
      }
    }
}

void fier_unpack_meta(const fier_config* cfg, const uint32_t* kmeta_host, uint16_t* s_host, uint16_t* z_host) {
  if (check_cfg(cfg) != FIER_OK || !kmeta_host || !s_host || !z_host) return;
  const size_t n = (size_t)units_of(cfg) * (size_t)(cfg->max_ctx / cfg->group_size) * kD;
  for (size_t i = 0; i < n; ++i) {
    s_host[i] = (uint16_t)(kmeta_host[i] & 0xffffu);
    z_host[i] = (uint16_t)(kmeta_host[i] >> 16);
  }
}

}  // extern "C"
