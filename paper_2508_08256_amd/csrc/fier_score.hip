// The scoring kernel (Alg. 1 step 2; with the histogram and the append: first kernel of the fused step) and its
// launcher.  The device code is in fier_score_dev.h (the one-launch step runs the same body in its own kernel).
#include "fier_score_dev.h"

namespace fier {

template <int DT, int NREP, bool HIST>
__global__ __launch_bounds__(256) void score_kernel(const ScoreArgs sa) {
  __shared__ uint32_t lhist[HIST ? kSelBins : 1];
  __shared__ __attribute__((aligned(16))) unsigned char a_lds[kScoreLdsA];
  // The workgroup's scores wait here and leave as one contiguous burst at the end: stores interleaved block by block
  // with the loads make the memory turn around between reading and writing all the time.
  __shared__ __attribute__((aligned(16))) float lscore[kScoreMaxBpw * 4 * kPair];
  score_body<DT, NREP, HIST, false>(sa, (int)blockIdx.x, (int)gridDim.x, lhist, a_lds, lscore);
}

// The kernel arguments of a scoring launch (shared with the one-launch step); false if the shape does not fit.
bool fill_score_args(ScoreArgs& sa, KvLayout lay, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                     const void* q, const int32_t* seq_lens, int extra, float* scores, const StepBuffers* sb, void* K,
                     void* V, const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                     int group_size, bool hist, int* rounds_out) {
  sa.kbits = (const uint4*)kbits;
  sa.kmeta = (const uint4*)kmeta;
  sa.kabsmax = kabsmax;
  sa.q = (const uint16_t*)q;
  sa.seq_lens = seq_lens;
  sa.extra = extra;
  sa.scores = scores;
  sa.ctl = sb ? sb->ctl : nullptr;
  sa.ghist = sb ? sb->hist : nullptr;
  sa.K = (uint32_t*)K;
  sa.V = (uint32_t*)V;
  sa.k_new = (const uint32_t*)k_new;
  sa.v_new = (const uint32_t*)v_new;
  sa.newmax = sb ? sb->newmax : nullptr;
  sa.n_kv_heads = n_kv_heads;
  sa.max_ctx = max_ctx;
  sa.gshift = group_size == 256 ? 3 : group_size == 128 ? 2 : group_size == 64 ? 1 : 0;
  sa.bpw = score_blocks_per_wave(units, max_ctx, hist, rounds_out);
  const int n_blocks = (max_ctx + kPair - 1) / kPair;
  sa.n_x = (n_blocks + 4 * sa.bpw - 1) / (4 * sa.bpw);  // scoring workgroups per unit
  sa.no_arrival = 0;
  sa.lay = lay;
  return sa.bpw <= kScoreMaxBpw;  // always: at most 12, + 1
}

template <int DT, bool HIST>
static hipError_t launch_score_dt(KvLayout lay, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                                  const void* q, const int32_t* seq_lens, int extra, float* scores,
                                  const StepBuffers* sb, const int32_t* budgets, int max_budget, void* K, void* V,
                                  const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                                  int group_size, hipStream_t st) {
  ScoreArgs sa;
  if (!fill_score_args(sa, lay, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, sb, K, V, k_new, v_new, units,
                       n_kv_heads, max_ctx, group_size, HIST))
    return hipErrorInvalidValue;
  dim3 grid((unsigned)units * (unsigned)(sa.n_x + (HIST ? 1 : 0)));
#define FIER_SCORE_CASE(R)                                \
  case R:                                                 \
    score_kernel<DT, R, HIST><<<grid, 256, 0, st>>>(sa);  \
    break;
  switch (n_rep) {
    FIER_SCORE_CASE(1)
    FIER_SCORE_CASE(2)
    FIER_SCORE_CASE(3)
    FIER_SCORE_CASE(4)
    FIER_SCORE_CASE(5)
    FIER_SCORE_CASE(6)
    FIER_SCORE_CASE(7)
    FIER_SCORE_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_SCORE_CASE
  return hipGetLastError();
}

hipError_t launch_score(int dtype, KvLayout lay, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                        const void* q, const int32_t* seq_lens, int extra, float* scores, const StepBuffers* sb,
                        const int32_t* budgets, int max_budget, void* K, void* V, const void* k_new,
                        const void* v_new, int units, int n_kv_heads, int max_ctx, int group_size, hipStream_t st) {
  if (sb) {
    if (dtype == DT_F16)
      return launch_score_dt<DT_F16, true>(lay, n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, sb, budgets,
                                           max_budget, K, V, k_new, v_new, units, n_kv_heads, max_ctx, group_size, st);
    return launch_score_dt<DT_BF16, true>(lay, n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, sb, budgets,
                                          max_budget, K, V, k_new, v_new, units, n_kv_heads, max_ctx, group_size, st);
  }
  if (dtype == DT_F16)
    return launch_score_dt<DT_F16, false>(lay, n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, nullptr, nullptr,
                                          0, nullptr, nullptr, nullptr, nullptr, units, n_kv_heads, max_ctx, group_size, st);
  return launch_score_dt<DT_BF16, false>(lay, n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, nullptr, nullptr, 0,
                                         nullptr, nullptr, nullptr, nullptr, units, n_kv_heads, max_ctx, group_size, st);
}

}  // namespace fier
