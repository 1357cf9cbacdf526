/*
 * libfier -- the decode hot path of Fier (arxiv 2508.08256, "token-level KV retrieval
 * via 1-bit quantization") for one AMD MI355X (gfx950).
 *
 * One decode step of one attention layer, per (batch element, kv head) "unit":
 *   1. keep a 1-bit copy of the key cache, group size g = 32 tokens per channel, with
 *      one (s, z) pair per group and channel                     (Alg. 1 step 1, Eq. 5)
 *   2. score every cached token: q . dequant(1-bit key)           (Alg. 1 step 2)
 *   3. pick the top-B tokens per kv head                          (Alg. 1 step 3)
 *   4. exact softmax attention over the selected K/V rows only    (Alg. 1 step 4)
 *
 * General rules of this ABI
 *   - Plain C.  Every pointer in fier_cache and every pointer argument documented as
 *     "device" is device memory owned by the caller; the library allocates nothing,
 *     keeps no state between calls and never frees.  "host" pointers are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and never synchronise; results are valid once the stream has been
 *     synchronised by the caller.  Calls that touch the same buffers must be ordered by
 *     the caller (same stream, or events).
 *   - Every device pointer must be 16-byte aligned, a workspace 256-byte aligned (FIER_EALIGN otherwise).
 *   - Arguments are validated on the host before anything is launched; on any error
 *     nothing has been enqueued.  FIER_EHIP reports a failed launch: kernels launched before the failing
 *     one may already have run, and the workspace must then be zero-filled again before it is reused.
 *   - K, V, q, k_new and v_new must be finite (no infinities, no NaNs): the quantizer's minimum / maximum,
 *     the score bound and the selection are defined on finite values only.
 *   - Units are ordered batch-major: u = b * n_kv_heads + h.  The query heads that
 *     share kv head h are h * n_rep .. h * n_rep + n_rep - 1, n_rep = n_q_heads / n_kv_heads.
 *
 * Data layout in device memory (D = head_dim = 128, g = group_size: 32 by default, or 64, 128, 256)
 *   k, v     [batch][n_kv_heads][max_ctx][D]     16-bit floats (binary16 or bfloat16)
 *   kbits    [units][max_ctx][4] uint32            one 128-bit code word (16 bytes) per token:
 *              bit i of word d holds channel c = 64 (d & 1) + 2 i + (d >> 1), i.e. words 0 / 1 carry
 *              the even channels 0..62 / 64..126 and words 2 / 3 the odd channels 1..63 / 65..127.
 *              Bits of tokens not present are 0.  A wavefront reads the 64 tokens of a "pair block"
 *              (two quantization groups when g = 32) as one coalesced 1 KiB request, lane = token.
 *   kmeta    [units][max_ctx / g][D] uint32       low half = s, high half = z of group
 *              (u, G, c), G = token / g, both in the K dtype: dequant(k) = z + bit * s.
 *   Together 16 + 512/g bytes per cached token and unit (32 for g = 32: 1/8 of a 16-bit key cache), the
 *   ratio (1 + 32/g)/16 of Eq. 8: 0.125, 0.078 and 0.070 for g = 32, 128 and 256 (Sec. 4.4 ablation).
 *   kabsmax  [units][D] float: max over the quantized tokens of max(|z|, |z + s|) per channel.  With
 *              it |score| <= R = sum_c |q_c| kabsmax_c is known before any score is computed, which
 *              lets the scoring kernel histogram its scores in the same pass (512 bytes per unit).
 *   seq_lens [batch] int32, device: tokens currently valid in each sequence.
 *
 * Workspace: device memory, 256-byte aligned, passed to every call that needs scratch as a pointer and its
 * size in bytes.  A call returns FIER_EWORKSPACE, before anything is launched, when the pointer is NULL or the
 * size is below fier_workspace_bytes(cfg, max_budget) for the max_budget the call works with (whole-cache
 * attention: max_ctx).  The caller zero-fills it ONCE after allocating it; every call leaves the counters
 * inside it zero again, so it can be reused by any later call with the same cfg (one call at a time).
 */
#ifndef FIER_H
#define FIER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FIER_OK = 0,
  FIER_EINVAL = -1,       /* null pointer, negative size, bad enum            */
  FIER_ESHAPE = -2,       /* head counts / context capacity not supported      */
  FIER_EALIGN = -3,       /* a device pointer is not 16-byte aligned            */
  FIER_EWORKSPACE = -4,   /* workspace missing or smaller than the call needs  */
  FIER_EUNSUPPORTED = -5, /* head_dim != 128, group_size not 32/64/128/256, n_rep > 8 */
  FIER_EHIP = -6          /* a kernel launch failed                             */
} fier_status;

typedef enum { FIER_F16 = 0, FIER_BF16 = 1 } fier_dtype;

typedef struct fier_config {
  int32_t n_q_heads;  /* multiple of n_kv_heads, n_rep = n_q_heads / n_kv_heads <= 8 */
  int32_t n_kv_heads;
  int32_t head_dim;   /* 128 */
  int32_t group_size; /* tokens per quantization group along each channel: 32, 64, 128 or 256; divides max_ctx */
  int32_t max_ctx;    /* row capacity of every unit's cache; multiple of 64, <= 2^20 */
  int32_t batch;
  int32_t kv_dtype;   /* fier_dtype of k, v, q, k_new, v_new and of (s, z)           */
  float sm_scale;     /* softmax scale of step 4, e.g. 1/sqrt(head_dim)              */
} fier_config;

typedef struct fier_cache { /* one layer; all pointers device, caller-owned */
  void *k; /* block_table == NULL: [units][max_ctx][head_dim], unit = sequence * n_kv_heads + kv head.      */
  void *v; /* block_table != NULL: a pool [pool blocks][n_kv_heads][block_tokens][head_dim]                 */
  uint32_t *kbits;         /* fier_packed_bits_bytes(cfg) bytes */
  uint32_t *kmeta;         /* fier_packed_meta_bytes(cfg) bytes */
  float *kabsmax;          /* [units][D]: per channel, an upper bound of |dequantized key| over the
                              tokens quantized so far; written by fier_quantize_keys, raised by appends.  A cache
                              that is filled by appends alone (no fier_quantize_keys call) must start with it
                              zero-filled */
  const int32_t *seq_lens; /* [batch] */
  /* Paged K / V rows (optional).  block_table is [batch][max_ctx / block_tokens]: entry j of sequence b is
   * the pool block that holds its tokens [j * block_tokens, (j + 1) * block_tokens), for all kv heads.
   * Entries that cover tokens < seq_len (+ the appended one) must be valid pool block numbers: the kernels
   * cannot check them; later entries may be loaded but are never used.  k and v share the table.  block_tokens is a power of
   * two >= max(64, group_size) that divides max_ctx, else FIER_ESHAPE; NULL with block_tokens = 0 selects
   * the contiguous layout (block_tokens != 0 with a NULL table: FIER_EINVAL).  The packed 1-bit cache
   * (kbits, kmeta, kabsmax), the scores and every index are per unit and contiguous in both layouts, so
   * results are bit-identical whichever layout holds the rows. */
  const int32_t *block_table;
  int32_t block_tokens;
} fier_cache;

/* Sizes (host only, no GPU needed).  0 if cfg is invalid. */
size_t fier_packed_bits_bytes(const fier_config *cfg);
size_t fier_packed_meta_bytes(const fier_config *cfg);
/* Scratch needed by fier_sparse_attn / fier_dense_attn / fier_decode_step for selections of at
 * most max_budget tokens per unit (fier_dense_attn: pass max_budget = max_ctx). */
size_t fier_workspace_bytes(const fier_config *cfg, int32_t max_budget);
/* For inspection: the byte offset inside such a workspace of the scores [units][max_ctx] float that the latest
 * fier_decode_step on it computed for its last layer (Alg. 1 step 2 as the fused step evaluates it).  0 if invalid. */
size_t fier_workspace_scores_offset(const fier_config *cfg, int32_t max_budget);
const char *fier_status_string(int status);
/* Check cfg alone: FIER_OK or the error the other calls would return for it. */
int fier_check_config(const fier_config *cfg);

/*
 * Alg. 1 step 1 (Eq. 5 as 1-bit round-to-nearest, Sec. 3.3).  For every unit, quantize tokens
 * [0, seq_len): per group of 32 consecutive tokens of a channel, z = the smallest element
 * (-0 stored as +0), s = (largest - z) rounded once to the K dtype (held at the largest finite
 * value on overflow), bit = 1 iff 2 * (k - z) >= s, all three evaluated in binary32.  A partial
 * last group uses the tokens present.  Writes every pair block that holds a valid token, and
 * the (s, z) of both of its groups (zeros for a group with no token); the rest is untouched.
 */
int fier_quantize_keys(const fier_config *cfg, const fier_cache *cache, void *stream);

/*
 * Sec. 3.1 decode-stage append.  For every unit write k_new / v_new ([batch][n_kv_heads][D],
 * device) into row seq_len of k / v, then re-derive the (s, z) and the bits of the group that
 * row falls in from the keys present (rows 32*floor(seq_len/32) .. seq_len).  After the call the
 * packed state equals fier_quantize_keys over seq_len + 1 tokens, bit for bit.  seq_lens is not
 * modified (the caller increments it); a unit with seq_len >= max_ctx is left unchanged.
 */
int fier_append_key(const fier_config *cfg, const fier_cache *cache, const void *k_new,
                    const void *v_new, void *stream);

/*
 * Alg. 1 step 2.  scores[u][j] = sum over the unit's n_rep query heads of q_r . (z + bit * s)
 * for j < seq_len + extra_tokens, binary32, unscaled.  q is [batch][n_q_heads][D] device;
 * scores is [units][max_ctx] device; entries at and past the scored length are not written.
 * extra_tokens is 0, or 1 to include a row appended in this step.
 */
int fier_score(const fier_config *cfg, const fier_cache *cache, const void *q, int32_t extra_tokens,
               float *scores, void *stream);

/*
 * Alg. 1 step 3.  Per unit: the min(budget, len) tokens of largest score among the first
 * len = seq_lens[b] + extra_tokens; equal scores go to the lower token index (-0 == +0);
 * indices are written in ascending order to idx[u][0 .. count[u]).  budgets is [batch] device
 * (values < 1 select nothing), max_budget is the row pitch of idx (host value >= every budget;
 * larger budgets are clamped to it).  Scores must be finite.  No workspace is used.
 */
int fier_topk(const fier_config *cfg, const float *scores, const int32_t *seq_lens,
              int32_t extra_tokens, const int32_t *budgets, int32_t max_budget, int32_t *idx,
              int32_t *count, void *stream);

/*
 * The same selection as fier_topk, bit for bit, computed by many workgroups per unit where a unit's scores do
 * not fit the registers of one (contexts beyond 36864 tokens: four small kernels instead of one workgroup per
 * unit streaming its scores four times; shorter contexts take fier_topk's kernel).  workspace:
 * fier_workspace_bytes(cfg, max_budget) bytes, the same one the other calls use.  max_budget is the row pitch
 * of idx as in fier_topk.
 */
int fier_topk_ws(const fier_config *cfg, const float *scores, const int32_t *seq_lens,
                 int32_t extra_tokens, const int32_t *budgets, int32_t max_budget, int32_t *idx,
                 int32_t *count, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Alg. 1 step 4.  For every query head: p = softmax(sm_scale * q . K[S]^T), out = p V[S], with
 * S = idx[u][0 .. count[u]) (rows of this unit's cache, any order; an entry outside [0, max_ctx) is skipped).  Inputs are
 * read in the K dtype, logits, softmax and the output are binary32.  out is
 * [batch][n_q_heads][D] float, device.  count[u] == 0 gives zeros.
 */
int fier_sparse_attn(const fier_config *cfg, const fier_cache *cache, const void *q,
                     const int32_t *idx, const int32_t *count, int32_t max_budget, float *out,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Sec. 3.1 full-cache decode attention softmax(sm_scale * q K^T) V over rows [0, seq_len +
 * extra_tokens): the "Full KV" comparison of Sec. 4.5, same kernels as step 4 without the gather.
 * workspace: fier_workspace_bytes(cfg, max_ctx). */
int fier_dense_attn(const fier_config *cfg, const fier_cache *cache, const void *q,
                    int32_t extra_tokens, float *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One whole decode step (Alg. 1 with the append of Sec. 3.1) for n_layers layers, one enqueue:
 * for each layer l: append k_new[l] / v_new[l] (skipped if k_new is NULL), score all
 * seq_len (+1 if appended) tokens, select the top budgets[b], attend over the selection.
 *   layers   [n_layers] host array of fier_cache (device pointers inside)
 *   q        [n_layers][batch][n_q_heads][D] device;   k_new, v_new [n_layers][batch][n_kv_heads][D]
 *   out      [n_layers][batch][n_q_heads][D] float device
 *   idx_out / count_out   optional (NULL): [n_layers][units][max_budget] / [n_layers][units], the
 *            selection of every layer, for inspection
 *   workspace  fier_workspace_bytes(cfg, max_budget) bytes, reused by every layer
 * seq_lens are not modified.  A sequence whose cache is full (seq_len >= max_ctx) is not appended
 * to: the step works on its max_ctx rows as if k_new were NULL for it.
 */
int fier_decode_step(const fier_config *cfg, const fier_cache *layers, int32_t n_layers, const void *q,
                     const void *k_new, const void *v_new, const int32_t *budgets, int32_t max_budget,
                     float *out, int32_t *idx_out, int32_t *count_out, void *workspace, size_t workspace_bytes,
                     void *stream);

/*
 * fier_decode_step for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, serving loops and harnesses that forbid allocation): the scratch is a fixed 48 MiB array inside the
 * library's device image, one copy per GPU, held until the process ends.  Same arguments and results as
 * fier_decode_step without the workspace.  Returns FIER_EWORKSPACE, with nothing enqueued, when
 * fier_workspace_bytes(cfg, max_budget) exceeds 48 MiB (e.g. 32 units of 131072 tokens fit, 128 units of 65536 do
 * not).  The call allocates nothing and never synchronises; it clears the part of the array that must start at zero
 * with a small kernel on `stream`, so it can be captured into a graph.  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (different streams, different threads) race; order them.
 */
int fier_decode_step_static(const fier_config *cfg, const fier_cache *layers, int32_t n_layers, const void *q,
                            const void *k_new, const void *v_new, const int32_t *budgets, int32_t max_budget,
                            float *out, int32_t *idx_out, int32_t *count_out, void *stream);

/*
 * The deployment policy of Sec. 4.1 (the method is not applied to the first two layers): as fier_decode_step,
 * except that every layer l with dense_layers[l] != 0 (HOST array of n_layers bytes; NULL = no such layer) runs
 * full attention over all seq_len (+ 1) rows after its append; its packed cache is still kept up to date.  For
 * those layers idx_out and count_out are not written.  If any layer is dense the workspace must have
 * fier_workspace_bytes(cfg, max_ctx) bytes.
 */
int fier_decode_step_mixed(const fier_config *cfg, const fier_cache *layers, int32_t n_layers,
                           const uint8_t *dense_layers, const void *q, const void *k_new, const void *v_new,
                           const int32_t *budgets, int32_t max_budget, float *out, int32_t *idx_out,
                           int32_t *count_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One kernel of fier_decode_step alone, for measurement and tests.  After the first kernel (phase 1: append + score +
 * score histogram) the step takes one of two forms, chosen from cfg, max_budget and whether idx_out is given;
 * fier_decode_step_kernels returns the number of kernels of the form a call gets (not counting the optional
 * index-list kernel; with_index_list != 0: a call with idx_out), 0 for an invalid configuration:
 *   2 kernels, with one or two query heads per kv head; with more of them if idx_out is null and the second kernel
 *     has at most twice the workgroups the GPU holds at once: phase 2 = exact threshold + attention over the selected
 *     rows + merge in one launch; phase 3 = the ascending index list (launched by the step only if idx_out is given;
 *     may be repeated);
 *   3 kernels otherwise: phase 2 = exact threshold, phase 3 = selection + attention + merge, which also writes
 *     idx_out (may be repeated).
 * Same arguments as fier_decode_step.  Phase p works on what phases 1..p-1 of the latest step on this workspace and
 * these layers left behind, so the sequence 1, 2, 3 equals fier_decode_step.  Phase 1 adds its scores to the
 * workspace's histograms and phase 2 consumes and clears them: phase 1 may be repeated for timing (follow it with one
 * phase 2 before the next real step), phase 2 only after a phase 1.  Phases 2 + 16 f and 3 + 16 f, f = 1..3, are for
 * tests: the two-kernel form whatever the shape, its second kernel with flags f (1: no workgroup picks up the
 * threshold itself, the merging workgroup attends over all threshold-bin rows; 2: checksums of the attended rows in
 * the control blocks); phases 2 + 64 and 3 + 64: the three-kernel form whatever the shape.
 */
int fier_decode_step_kernels(const fier_config *cfg, int32_t max_budget, int32_t with_index_list);
int fier_decode_step_phase(const fier_config *cfg, const fier_cache *layers, int32_t n_layers, const void *q,
                           const void *k_new, const void *v_new, const int32_t *budgets, int32_t max_budget,
                           float *out, int32_t *idx_out, int32_t *count_out, void *workspace,
                           size_t workspace_bytes, int32_t phase, void *stream);

/*
 * Page-level importance, the page-retrieval baseline the paper compares with (Sec. 3.2, Eq. 1-3) and the
 * "averaged quantized score per page" ablation of Sec. 4.4: a second workload for fier_topk and fier_sparse_attn.
 * A page = page_tokens (8, 16 or 32) consecutive tokens of a unit.
 *   page_meta [units][max_ctx / page_tokens][D] uint32, device: channel-wise minimum (low half) and maximum (high
 *   half) key of the page over the tokens present, in the K dtype; fier_page_meta_bytes bytes (512 per page: the
 *   load ratio 2 / page_tokens of the paper).
 * fier_page_minmax builds it from the K rows [0, seq_len); fier_page_append folds the row k_new
 * ([batch][n_kv_heads][D]) written at position seq_len into its page (call it next to fier_append_key).
 * fier_page_score: page_scores [units][max_ctx / page_tokens] float.  mode 0: max over the channels of
 * max(q_i kmax_i, q_i kmin_i), Eq. 3 as printed (exact); mode 1: the sum over the channels instead, an upper bound
 * of q . k for every key of the page.  Per-head page scores of the query heads of a kv head are added.  Pages without
 * tokens get -inf.
 * fier_page_mean_score: page score = average of the token scores (fier_score's output) over the page's tokens.
 * Selection: call fier_topk on page_scores with a fier_config whose max_ctx is max_ctx / page_tokens (a multiple of 64)
 * and a device array of page counts ceil(seq_len / page_tokens) as its seq_lens.
 * fier_expand_pages: idx [units][max_budget] = the tokens of the selected pages (page_idx [units][max_pages] ascending,
 * page_count [units]) in ascending order, clipped to seq_len + extra_tokens; count [units] = how many.
 */
size_t fier_page_meta_bytes(const fier_config *cfg, int32_t page_tokens);
int fier_page_minmax(const fier_config *cfg, const fier_cache *cache, int32_t page_tokens, uint32_t *page_meta,
                     void *stream);
int fier_page_append(const fier_config *cfg, const int32_t *seq_lens, int32_t page_tokens, const void *k_new,
                     uint32_t *page_meta, void *stream);
int fier_page_score(const fier_config *cfg, const uint32_t *page_meta, int32_t page_tokens, const int32_t *seq_lens,
                    int32_t extra_tokens, const void *q, int32_t mode, float *page_scores, void *stream);
int fier_page_mean_score(const fier_config *cfg, const float *scores, const int32_t *seq_lens, int32_t extra_tokens,
                         int32_t page_tokens, float *page_scores, void *stream);
int fier_expand_pages(const fier_config *cfg, const int32_t *page_idx, const int32_t *page_count, int32_t max_pages,
                      const int32_t *seq_lens, int32_t extra_tokens, int32_t page_tokens, int32_t *idx, int32_t *count,
                      int32_t max_budget, void *stream);

/* Host helpers for inspection: physical packed layout -> logical arrays, all host memory.
 * bits [units][max_ctx][D] one byte (0/1) per element; s, z [units][max_ctx/32][D] raw 16-bit words. */
void fier_unpack_bits(const fier_config *cfg, const uint32_t *kbits_host, uint8_t *bits_host);
void fier_unpack_meta(const fier_config *cfg, const uint32_t *kmeta_host, uint16_t *s_host,
                      uint16_t *z_host);

#ifdef __cplusplus
}
#endif
#endif /* FIER_H */
