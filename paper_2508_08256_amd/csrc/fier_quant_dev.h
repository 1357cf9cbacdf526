// The 1-bit group quantizer as a device function, shared by the bulk quantizer, the append kernel and the
// fused decode step (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3).
#pragma once

#include "fier_dev.h"

namespace fier {

struct GroupCode {          // what one lane (channels 2l, 2l+1) learns about a group
  uint32_t meta_lo, meta_hi;  // s | z << 16 in the K dtype
  float s_lo, z_lo, s_hi, z_hi;  // the same as binary32
  float amax_lo, amax_hi;     // max(|z|, |z + s|): the larger reconstruction level in magnitude
  uint32_t bits_lo, bits_hi;  // bit t = code of token t (channel-major view of the group)
};

// Quantize one group (ntok in [1, 32] tokens present) for the lane's two channels.
// rows[t] holds the packed pair (channel 2l in the low half) of token t; entries t >= ntok are ignored.
// Lane lane_base + t receives the 128-bit code word of token t in `mine` (zero for tokens not present):
// x, y = even channels 0..62 / 64..126 (bit i = channel 2i, 64 + 2i), z, w = odd channels likewise.
// The decision arithmetic is binary32 without contraction:  z = min (-0 -> +0);  s = RN_dtype(max - z), held at
// the largest finite value;  bit = 2 * (k - z) >= s.
template <int DT>
__device__ __forceinline__ void quantize_group(const uint32_t (&rows)[kG], int ntok, int lane, int lane_base,
                                               uint4& mine, GroupCode& gc) {
#pragma clang fp contract(off)
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
  const uint32_t s0 = f2w<DT>(d0), s1 = f2w<DT>(d1);
  const uint32_t z0 = f2w<DT>(mn0), z1 = f2w<DT>(mn1);
  const float sf0 = w2f<DT>(s0), sf1 = w2f<DT>(s1);
  const float zf0 = w2f<DT>(z0), zf1 = w2f<DT>(z1);
  uint32_t b0 = 0, b1 = 0;
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    float a = lo16f<DT>(rows[t]) - zf0;
    float b = hi16f<DT>(rows[t]) - zf1;
    bool present = t < ntok;
    const bool c0 = present && (a + a >= sf0), c1 = present && (b + b >= sf1);
    const uint64_t even = __ballot(c0);
    const uint64_t odd = __ballot(c1);
    b0 |= c0 ? (1u << t) : 0u;
    b1 |= c1 ? (1u << t) : 0u;
    if (lane == lane_base + t)
      mine = make_uint4((uint32_t)even, (uint32_t)(even >> 32), (uint32_t)odd, (uint32_t)(odd >> 32));
  }
  gc.meta_lo = s0 | (z0 << 16);
  gc.meta_hi = s1 | (z1 << 16);
  gc.s_lo = sf0;
  gc.z_lo = zf0;
  gc.s_hi = sf1;
  gc.z_hi = zf1;
  gc.amax_lo = fmaxf(fabsf(zf0), fabsf(zf0 + sf0));
  gc.amax_hi = fmaxf(fabsf(zf1), fabsf(zf1 + sf1));
  gc.bits_lo = b0;
  gc.bits_hi = b1;
}

// kabsmax[u][c] >= |dequantized key| of every token quantized so far: raised with an integer max on the bit
// pattern (non-negative floats order like unsigned integers); a plain read filters most of the atomics.
__device__ __forceinline__ void raise_absmax(float* __restrict__ slot, float a) {
  if (a > *reinterpret_cast<volatile float*>(slot)) atomicMax(reinterpret_cast<unsigned int*>(slot), __float_as_uint(a));
}

// One wavefront appends row L of a unit (lane = channel pair): writes the K/V rows, re-derives the group the row
// falls in from the rows present (the new row comes from registers) and stores its code words and (s, z).
// Returns the group's code in gc; t0 = first token of the group, ntok = tokens now present in it.
template <int DT>
__device__ __forceinline__ void append_row(uint32_t* __restrict__ K, uint32_t* __restrict__ V,
                                           uint32_t* __restrict__ kbits, uint32_t* __restrict__ kmeta, int unit,
                                           int L, int max_ctx, uint32_t kn, uint32_t vn, int lane, GroupCode& gc,
                                           int& t0, int& ntok) {
  const int n_groups = max_ctx / kG;
  K[((size_t)unit * max_ctx + L) * (kD / 2) + lane] = kn;
  V[((size_t)unit * max_ctx + L) * (kD / 2) + lane] = vn;
  const int Gi = L / kG;
  t0 = Gi * kG;
  ntok = L - t0 + 1;
  uint32_t rows[kG];
  const uint32_t* src = K + ((size_t)unit * max_ctx + t0) * (kD / 2) + lane;
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    // rows before the new one come from memory (t0 + t < L: never the row written above)
    uint32_t r = t < ntok - 1 ? src[(size_t)t * (kD / 2)] : 0u;
    rows[t] = (t == ntok - 1) ? kn : r;
  }
  uint4 mine = make_uint4(0, 0, 0, 0);
  quantize_group<DT>(rows, ntok, lane, 0, mine, gc);
  uint4* bdst = reinterpret_cast<uint4*>(kbits) + (size_t)unit * max_ctx + t0;
  uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi) * kD) + lane;
  *mdst = make_uint2(gc.meta_lo, gc.meta_hi);
  const bool opens_pair_block = (Gi & 1) == 0 && ntok == 1;  // its second group holds no token yet
  if (lane < kG || opens_pair_block) bdst[lane] = mine;
  if (opens_pair_block) {
    uint2* mdst1 = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi + 1) * kD) + lane;
    *mdst1 = make_uint2(0, 0);
  }
}

}  // namespace fier
