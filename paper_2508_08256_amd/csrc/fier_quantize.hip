// 1-bit group quantizer of the key cache (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3)
// and the decode-stage append of Sec. 3.1.
//
// One wavefront owns one pair block (64 tokens = two groups of 32).  Lane l owns channels 2l and 2l+1:
// every row read is one fully coalesced 256-byte request, the min/max over the 32 tokens of a group
// never leaves the lane's registers, and the lane ends up holding exactly the four 32-bit words
// (2 channels x 2 groups) that are adjacent in the packed layout -> one 16-byte store per lane.
//
// The decision arithmetic is fixed so that any implementation of the same definition produces the
// same bits:  z = min (an input value, -0 -> +0);  s = RN_dtype(f32(max) - f32(z)), held at the
// largest finite value;  bit = 2*(f32(k) - f32(z)) >= f32(s);  all in binary32, no contraction.
#include "fier_dev.h"
#include "fier_kernels.h"

#pragma clang fp contract(off)

namespace fier {

// Quantize one group (ntok in [1, 32] tokens present) for the lane's two channels.
// rows[t] holds the packed pair (channel 2l in the low half) of token t; entries t >= ntok are ignored.
template <int DT>
__device__ __forceinline__ void quantize_group(const uint32_t (&rows)[kG], int ntok, uint32_t& word_lo,
                                               uint32_t& word_hi, uint32_t& meta_lo, uint32_t& meta_hi) {
  float mn0 = lo16f<DT>(rows[0]), mx0 = mn0;
  float mn1 = hi16f<DT>(rows[0]), mx1 = mn1;
#pragma unroll
  for (int t = 1; t < kG; ++t) {
    float a = lo16f<DT>(rows[t]);
    float b = hi16f<DT>(rows[t]);
    bool present = t < ntok;
    mn0 = (present && a < mn0) ? a : mn0;
    mx0 = (present && a > mx0) ? a : mx0;
    mn1 = (present && b < mn1) ? b : mn1;
    mx1 = (present && b > mx1) ? b : mx1;
  }
  const float cap = DT == DT_F16 ? 65504.0f : 3.3895313892515355e38f;
  if (mn0 == 0.0f) mn0 = 0.0f;
  if (mn1 == 0.0f) mn1 = 0.0f;
  float d0 = mx0 - mn0;
  float d1 = mx1 - mn1;
  d0 = d0 > cap ? cap : d0;
  d1 = d1 > cap ? cap : d1;
  if (d0 == 0.0f) d0 = 0.0f;
  if (d1 == 0.0f) d1 = 0.0f;
  uint32_t s0 = f2w<DT>(d0), s1 = f2w<DT>(d1);
  uint32_t z0 = f2w<DT>(mn0), z1 = f2w<DT>(mn1);
  float sf0 = w2f<DT>(s0), sf1 = w2f<DT>(s1);
  float zf0 = w2f<DT>(z0), zf1 = w2f<DT>(z1);
  uint32_t w0 = 0, w1 = 0;
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    float a = lo16f<DT>(rows[t]) - zf0;
    float b = hi16f<DT>(rows[t]) - zf1;
    bool present = t < ntok;
    w0 |= (present && (a + a >= sf0)) ? (1u << t) : 0u;
    w1 |= (present && (b + b >= sf1)) ? (1u << t) : 0u;
  }
  word_lo = w0;
  word_hi = w1;
  meta_lo = s0 | (z0 << 16);
  meta_hi = s1 | (z1 << 16);
}

// grid (ceil(n_pairs / 4), units), block 256: wave w of block x owns pair block 4x + w.
template <int DT>
__global__ __launch_bounds__(256) void quantize_kernel(const uint32_t* __restrict__ K, uint32_t* __restrict__ kbits,
                                                       uint32_t* __restrict__ kmeta,
                                                       const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                       int max_ctx) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int unit = blockIdx.y;
  const int P = blockIdx.x * 4 + wave;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  if (P * kPair >= L) return;
  const int n_pairs = max_ctx / kPair;
  const int n_groups = max_ctx / kG;
  uint32_t words[2][2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int t0 = P * kPair + h * kG;
    int ntok = L - t0;
    ntok = ntok > kG ? kG : ntok;
    uint32_t meta0 = 0, meta1 = 0;
    words[h][0] = 0;
    words[h][1] = 0;
    if (ntok > 0) {
      uint32_t rows[kG];
      const uint32_t* src = K + ((size_t)unit * max_ctx + t0) * (kD / 2) + lane;
#pragma unroll
      for (int t = 0; t < kG; ++t) rows[t] = src[(size_t)(t < ntok ? t : 0) * (kD / 2)];
      quantize_group<DT>(rows, ntok, words[h][0], words[h][1], meta0, meta1);
    }
    uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + 2 * P + h) * kD) + lane;
    *mdst = make_uint2(meta0, meta1);
  }
  uint4* bdst = reinterpret_cast<uint4*>(kbits + ((size_t)unit * n_pairs + P) * (kD * 2)) + lane;
  *bdst = make_uint4(words[0][0], words[1][0], words[0][1], words[1][1]);
}

// grid (units), block 64: one wavefront per unit.  Writes the new K/V rows at position L = seq_len and
// re-derives the group that row falls in from the rows present (the new row comes from registers).
template <int DT>
__global__ __launch_bounds__(64) void append_kernel(uint32_t* __restrict__ K, uint32_t* __restrict__ V,
                                                    uint32_t* __restrict__ kbits, uint32_t* __restrict__ kmeta,
                                                    const int32_t* __restrict__ seq_lens,
                                                    const uint32_t* __restrict__ k_new,
                                                    const uint32_t* __restrict__ v_new, int n_kv_heads, int max_ctx) {
  const int lane = threadIdx.x;
  const int unit = blockIdx.x;
  const int L = seq_lens[unit / n_kv_heads];
  if (L < 0 || L >= max_ctx) return;
  const int n_pairs = max_ctx / kPair;
  const int n_groups = max_ctx / kG;
  const uint32_t kn = k_new[(size_t)unit * (kD / 2) + lane];
  const uint32_t vn = v_new[(size_t)unit * (kD / 2) + lane];
  K[((size_t)unit * max_ctx + L) * (kD / 2) + lane] = kn;
  V[((size_t)unit * max_ctx + L) * (kD / 2) + lane] = vn;
  const int Gi = L / kG;
  const int t0 = Gi * kG;
  const int ntok = L - t0 + 1;
  uint32_t rows[kG];
  const uint32_t* src = K + ((size_t)unit * max_ctx + t0) * (kD / 2) + lane;
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    uint32_t r = src[(size_t)(t < ntok - 1 ? t : 0) * (kD / 2)];
    rows[t] = (t == ntok - 1) ? kn : r;
  }
  if (ntok == 1) rows[0] = kn;
  uint32_t w0, w1, m0, m1;
  quantize_group<DT>(rows, ntok, w0, w1, m0, m1);
  const int P = Gi >> 1, h = Gi & 1;
  uint32_t* bdst = kbits + ((size_t)unit * n_pairs + P) * (kD * 2) + 4 * lane;
  bdst[h] = w0;
  bdst[2 + h] = w1;
  uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi) * kD) + lane;
  *mdst = make_uint2(m0, m1);
  if (h == 0 && ntok == 1) {  // first token of a new pair block: its second group holds no token yet
    bdst[1] = 0;
    bdst[3] = 0;
    uint2* mdst1 = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi + 1) * kD) + lane;
    *mdst1 = make_uint2(0, 0);
  }
}

hipError_t launch_quantize(int dtype, const void* K, uint32_t* kbits, uint32_t* kmeta, const int32_t* seq_lens,
                           int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  dim3 grid((max_ctx / kPair + 3) / 4, units);
  if (dtype == DT_F16)
    quantize_kernel<DT_F16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, seq_lens, n_kv_heads, max_ctx);
  else
    quantize_kernel<DT_BF16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, seq_lens, n_kv_heads, max_ctx);
  return hipGetLastError();
}

hipError_t launch_append(int dtype, void* K, void* V, uint32_t* kbits, uint32_t* kmeta, const int32_t* seq_lens,
                         const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                         hipStream_t st) {
  if (dtype == DT_F16)
    append_kernel<DT_F16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, seq_lens,
                                                (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx);
  else
    append_kernel<DT_BF16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, seq_lens,
                                                 (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx);
  return hipGetLastError();
}

}  // namespace fier
