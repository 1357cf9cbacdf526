// Approximate scores from the 1-bit key cache (Alg. 1 step 2):
//   score[j] = sum_c q_c * (z[G(j)][c] + bit[j][c] * s[G(j)][c]),  q = sum of the unit's query heads.
//
// Lane = token.  One wavefront owns one pair block (64 tokens = groups 2P and 2P+1):
//   * the 64-bit word pair of channel c is exactly the wavefront's lane mask "bit c of my token is 1";
//     it is fetched with scalar loads (the address is uniform) and used as a select mask;
//   * the per-group weights w[c] = q_c * s[G][c] differ between the two halves of the wavefront.  They are
//     kept distributed: each row of 16 lanes holds all 128 weights of its own group in 8 registers
//     (lane n of the row holds 8 channels), and a DPP row broadcast inside the select instruction hands
//     weight (m, n) to the 16 lanes of the row.  No LDS, no replication through memory;
//   * base[G] = sum_c q_c * z[G][c] is reduced inside each row with DPP rotates.
// Per (token, channel) this is one select (v_cndmask with DPP source) and one add.
//
// Channel <-> (register m, lane n) map: lane n of a row loads (s,z) of channels 4n..4n+3 and 64+4n..64+4n+3
// as two 16-byte requests: register m = 4*(c / 64) + (c % 4), lane n = (c % 64) / 4.
#include <utility>

#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

constexpr int kScorePairsPerWave = 4;  // pair blocks per wavefront -> 1024 tokens per 256-thread workgroup

typedef uint64_t mask8_t __attribute__((ext_vector_type(8)));

// Four consecutive channels (same broadcast lane BC, registers x0..x3 of one half):
//   acc_j += bit_j(lane) ? x_j[row lane BC] : 0.
// Each mask is the wave-uniform 64-bit lane mask of one channel.  The select takes the row-broadcast
// weight as its DPP source where the (inverted) mask in VCC is clear, a zero register where it is set.
template <int BC>
__device__ __forceinline__ void select_add4(uint64_t m0, uint64_t m1, uint64_t m2, uint64_t m3, float x0, float x1,
                                            float x2, float x3, float zero, float (&acc)[4]) {
  float t0, t1;
  asm("s_not_b64 vcc, %[m0]\n\t"
      "v_cndmask_b32_dpp %[t0], %[x0], %[z], vcc row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "s_not_b64 vcc, %[m1]\n\t"
      "v_cndmask_b32_dpp %[t1], %[x1], %[z], vcc row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_add_f32 %[a0], %[a0], %[t0]\n\t"
      "s_not_b64 vcc, %[m2]\n\t"
      "v_cndmask_b32_dpp %[t0], %[x2], %[z], vcc row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_add_f32 %[a1], %[a1], %[t1]\n\t"
      "s_not_b64 vcc, %[m3]\n\t"
      "v_cndmask_b32_dpp %[t1], %[x3], %[z], vcc row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_add_f32 %[a2], %[a2], %[t0]\n\t"
      "v_add_f32 %[a3], %[a3], %[t1]"
      : [t0] "=&v"(t0), [t1] "=&v"(t1), [a0] "+&v"(acc[0]), [a1] "+&v"(acc[1]), [a2] "+&v"(acc[2]),
        [a3] "+&v"(acc[3])
      : [m0] "s"(m0), [m1] "s"(m1), [m2] "s"(m2), [m3] "s"(m3), [x0] "v"(x0), [x1] "v"(x1), [x2] "v"(x2),
        [x3] "v"(x3), [z] "v"(zero), [bc] "n"(BC)
      : "vcc");
}

// channels C0 .. C0+7, whose eight 64-bit masks arrive as one 64-byte scalar load
template <int C0>
__device__ __forceinline__ void accumulate_8(const mask8_t mk, const float (&X)[8], float zero, float (&acc)[4]) {
  constexpr int H = 4 * (C0 / 64);
  constexpr int N = (C0 % 64) / 4;
  select_add4<N>(mk[0], mk[1], mk[2], mk[3], X[H], X[H + 1], X[H + 2], X[H + 3], zero, acc);
  select_add4<N + 1>(mk[4], mk[5], mk[6], mk[7], X[H], X[H + 1], X[H + 2], X[H + 3], zero, acc);
}

template <int B>
__device__ __forceinline__ void accumulate_all(const mask8_t* __restrict__ masks, mask8_t cur, const float (&X)[8],
                                               float zero, float (&acc)[4]) {
  if constexpr (B < 16) {
    mask8_t nxt = cur;
    if constexpr (B + 1 < 16) nxt = masks[B + 1];
    accumulate_8<8 * B>(cur, X, zero, acc);
    accumulate_all<B + 1>(masks, nxt, X, zero, acc);
  }
}

// grid (ceil(n_pairs / (4 * kScorePairsPerWave)), units), block 256.
template <int DT, int NREP>
__global__ __launch_bounds__(256) void score_kernel(const uint64_t* __restrict__ kbits,
                                                    const uint4* __restrict__ kmeta, const uint16_t* __restrict__ q,
                                                    const int32_t* __restrict__ seq_lens, int extra,
                                                    float* __restrict__ scores, int n_kv_heads, int max_ctx) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int unit = blockIdx.y;
  const int b = unit / n_kv_heads;
  int L = seq_lens[b] + extra;
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int n_pairs = max_ctx / kPair;
  const int n_groups = max_ctx / kG;
  const int row = lane >> 4, n = lane & 15;

  // the lane's 8 query channels, summed over the query heads that share this kv head (binary32)
  float qv[8];
  {
    const int h = unit - b * n_kv_heads;
    const uint16_t* qb = q + ((size_t)(b * n_kv_heads + h) * NREP) * kD;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int c = 64 * (m >> 2) + 4 * n + (m & 3);
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < NREP; ++r) s += w2f<DT>(qb[r * kD + c]);
      qv[m] = s;
    }
  }
  const float zero = 0.f;

#pragma unroll 1
  for (int i = 0; i < kScorePairsPerWave; ++i) {
    const int P = (blockIdx.x * kScorePairsPerWave + i) * 4 + wave;
    if (P * kPair >= L) break;
    const int Gl = 2 * P + (row >> 1);
    const uint4* mp = kmeta + ((size_t)unit * n_groups + Gl) * (kD / 4);
    const uint4 ma = mp[n];
    const uint4 mb = mp[16 + n];
    const uint32_t mw[8] = {ma.x, ma.y, ma.z, ma.w, mb.x, mb.y, mb.z, mb.w};
    float X[8];
    float basep = 0.f;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      X[m] = qv[m] * lo16f<DT>(mw[m]);
      basep += qv[m] * hi16f<DT>(mw[m]);
    }
    const float base = row_allsum(basep);
    // A DPP source must not be read within two issue slots of the VALU write that produced it.  The weights
    // pass through this fence so that every later DPP read of them is at least that far from their writes.
    asm volatile("s_nop 1"
                 : "+v"(X[0]), "+v"(X[1]), "+v"(X[2]), "+v"(X[3]), "+v"(X[4]), "+v"(X[5]), "+v"(X[6]), "+v"(X[7]));
    const uint64_t* masks = kbits + ((size_t)unit * n_pairs + P) * kD;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const mask8_t* m8 = reinterpret_cast<const mask8_t*>(masks);
    accumulate_all<0>(m8, m8[0], X, zero, acc);
    const float sc = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + base;
    const int tok = P * kPair + lane;
    if (tok < L) scores[(size_t)unit * max_ctx + tok] = sc;
  }
}

template <int DT>
static hipError_t launch_score_dt(int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const void* q,
                                  const int32_t* seq_lens, int extra, float* scores, int units, int n_kv_heads,
                                  int max_ctx, hipStream_t st) {
  const int n_pairs = max_ctx / kPair;
  dim3 grid((n_pairs + 4 * kScorePairsPerWave - 1) / (4 * kScorePairsPerWave), units);
#define FIER_SCORE_CASE(R)                                                                                     \
  case R:                                                                                                      \
    score_kernel<DT, R><<<grid, 256, 0, st>>>((const uint64_t*)kbits, (const uint4*)kmeta, (const uint16_t*)q, \
                                              seq_lens, extra, scores, n_kv_heads, max_ctx);                   \
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

hipError_t launch_score(int dtype, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const void* q,
                        const int32_t* seq_lens, int extra, float* scores, int units, int n_kv_heads, int max_ctx,
                        hipStream_t st) {
  if (dtype == DT_F16)
    return launch_score_dt<DT_F16>(n_rep, kbits, kmeta, q, seq_lens, extra, scores, units, n_kv_heads, max_ctx, st);
  return launch_score_dt<DT_BF16>(n_rep, kbits, kmeta, q, seq_lens, extra, scores, units, n_kv_heads, max_ctx, st);
}

}  // namespace fier
