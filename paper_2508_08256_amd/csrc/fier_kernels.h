// Internal launch interface between the C-ABI layer (fier_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fier {

constexpr int kAttnRowsSparse = 128;  // selected rows per workgroup of the split attention kernel
constexpr int kAttnRowsDense = 512;   // rows per workgroup when attending over the whole cache

hipError_t launch_quantize(int dtype, const void* K, uint32_t* kbits, uint32_t* kmeta, const int32_t* seq_lens,
                           int units, int n_kv_heads, int max_ctx, hipStream_t st);

hipError_t launch_append(int dtype, void* K, void* V, uint32_t* kbits, uint32_t* kmeta, const int32_t* seq_lens,
                         const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                         hipStream_t st);

hipError_t launch_score(int dtype, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const void* q,
                        const int32_t* seq_lens, int extra, float* scores, int units, int n_kv_heads, int max_ctx,
                        hipStream_t st);

hipError_t launch_topk(const float* scores, const int32_t* seq_lens, int extra, const int32_t* budgets,
                       int max_budget, int32_t* idx, int32_t* count, int units, int n_kv_heads, int max_ctx,
                       hipStream_t st);

// idx == nullptr: attend over rows [0, seq_len + extra) (dense).  rows_per_wg rows of the selection per
// workgroup; partials (po, pm, pl) hold n_splits entries per (unit, query head).
hipError_t launch_attn(int dtype, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                       const int32_t* count, const int32_t* seq_lens, int extra, int max_budget, int rows_per_wg,
                       int n_splits, float sm_scale, float* po, float* pm, float* pl, float* out, int units,
                       int n_kv_heads, int max_ctx, hipStream_t st);

}  // namespace fier
