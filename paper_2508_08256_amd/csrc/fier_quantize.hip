// 1-bit group quantizer of the key cache (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3)
// and the decode-stage append of Sec. 3.1.
//
// One wavefront owns one pair block (64 tokens = two groups of 32).  Lane l owns channels 2l and 2l+1:
// every row read is one fully coalesced 256-byte request and the min/max over the 32 tokens of a group
// never leaves the lane's registers.  The packed layout is token-major (16 bytes per token), so the
// channel-major decisions are transposed with wavefront ballots: the compare "bit of channel 2l (2l+1) of
// token t" over all 64 lanes IS the even (odd) 64-bit half of token t's code word; lane 32h+t keeps it,
// and after both groups every lane stores the 16 bytes of its own token -> one coalesced 1 KiB store.
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
// Lane lane_base + t receives the 128-bit code word of token t in `mine` (zero for tokens not present):
// x, y = even channels 0..62 / 64..126 (bit i = channel 2i, 64 + 2i), z, w = odd channels likewise.
template <int DT>
__device__ __forceinline__ void quantize_group(const uint32_t (&rows)[kG], int ntok, int lane, int lane_base,
                                               uint4& mine, uint32_t& meta_lo, uint32_t& meta_hi, float& amax_lo,
                                               float& amax_hi) {
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
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    float a = lo16f<DT>(rows[t]) - zf0;
    float b = hi16f<DT>(rows[t]) - zf1;
    bool present = t < ntok;
    const uint64_t even = __ballot(present && (a + a >= sf0));
    const uint64_t odd = __ballot(present && (b + b >= sf1));
    if (lane == lane_base + t) mine = make_uint4((uint32_t)even, (uint32_t)(even >> 32), (uint32_t)odd, (uint32_t)(odd >> 32));
  }
  meta_lo = s0 | (z0 << 16);
  meta_hi = s1 | (z1 << 16);
  // largest magnitude of the two reconstruction levels z and z + s
  amax_lo = fmaxf(amax_lo, fmaxf(fabsf(zf0), fabsf(zf0 + sf0)));
  amax_hi = fmaxf(amax_hi, fmaxf(fabsf(zf1), fabsf(zf1 + sf1)));
}

// kabsmax[u][c] >= |dequantized key| of every token quantized so far: raised with an integer max on the bit
// pattern (non-negative floats order like unsigned integers); a plain read filters most of the atomics.
__device__ __forceinline__ void raise_absmax(float* __restrict__ slot, float a) {
  if (a > *reinterpret_cast<volatile float*>(slot)) atomicMax(reinterpret_cast<unsigned int*>(slot), __float_as_uint(a));
}

// grid (ceil(n_pairs / 4), units), block 256: wave w of block x owns pair block 4x + w.
template <int DT>
__global__ __launch_bounds__(256) void quantize_kernel(const uint32_t* __restrict__ K, uint32_t* __restrict__ kbits,
                                                       uint32_t* __restrict__ kmeta, float* __restrict__ kabsmax,
                                                       const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                       int max_ctx) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int unit = blockIdx.y;
  const int P = blockIdx.x * 4 + wave;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  if (P * kPair >= L) return;
  const int n_groups = max_ctx / kG;
  uint4 mine = make_uint4(0, 0, 0, 0);
  float amax0 = 0.f, amax1 = 0.f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int t0 = P * kPair + h * kG;
    int ntok = L - t0;
    ntok = ntok > kG ? kG : ntok;
    uint32_t meta0 = 0, meta1 = 0;
    if (ntok > 0) {
      uint32_t rows[kG];
      const uint32_t* src = K + ((size_t)unit * max_ctx + t0) * (kD / 2) + lane;
#pragma unroll
      for (int t = 0; t < kG; ++t) rows[t] = src[(size_t)(t < ntok ? t : 0) * (kD / 2)];
      quantize_group<DT>(rows, ntok, lane, h * kG, mine, meta0, meta1, amax0, amax1);
    }
    uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + 2 * P + h) * kD) + lane;
    *mdst = make_uint2(meta0, meta1);
  }
  reinterpret_cast<uint4*>(kbits)[(size_t)unit * max_ctx + P * kPair + lane] = mine;
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, amax0);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, amax1);
}

__global__ void zero_absmax_kernel(float* __restrict__ kabsmax, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) kabsmax[i] = 0.f;
}

// grid (units), block 64: one wavefront per unit.  Writes the new K/V rows at position L = seq_len and
// re-derives the group that row falls in from the rows present (the new row comes from registers).
template <int DT>
__global__ __launch_bounds__(64) void append_kernel(uint32_t* __restrict__ K, uint32_t* __restrict__ V,
                                                    uint32_t* __restrict__ kbits, uint32_t* __restrict__ kmeta,
                                                    float* __restrict__ kabsmax,
                                                    const int32_t* __restrict__ seq_lens,
                                                    const uint32_t* __restrict__ k_new,
                                                    const uint32_t* __restrict__ v_new, int n_kv_heads, int max_ctx) {
  const int lane = threadIdx.x;
  const int unit = blockIdx.x;
  const int L = seq_lens[unit / n_kv_heads];
  if (L < 0 || L >= max_ctx) return;
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
  uint4 mine = make_uint4(0, 0, 0, 0);
  uint32_t m0, m1;
  float amax0 = 0.f, amax1 = 0.f;
  quantize_group<DT>(rows, ntok, lane, 0, mine, m0, m1, amax0, amax1);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, amax0);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, amax1);
  uint4* bdst = reinterpret_cast<uint4*>(kbits) + (size_t)unit * max_ctx + t0;
  uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi) * kD) + lane;
  *mdst = make_uint2(m0, m1);
  const bool opens_pair_block = (Gi & 1) == 0 && ntok == 1;  // its second group holds no token yet
  if (lane < kG || opens_pair_block) bdst[lane] = mine;
  if (opens_pair_block) {
    uint2* mdst1 = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi + 1) * kD) + lane;
    *mdst1 = make_uint2(0, 0);
  }
}

hipError_t launch_quantize(int dtype, const void* K, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                           const int32_t* seq_lens, int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  zero_absmax_kernel<<<(units * kD + 255) / 256, 256, 0, st>>>(kabsmax, units * kD);
  dim3 grid((max_ctx / kPair + 3) / 4, units);
  if (dtype == DT_F16)
    quantize_kernel<DT_F16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, n_kv_heads,
                                                  max_ctx);
  else
    quantize_kernel<DT_BF16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, n_kv_heads,
                                                   max_ctx);
  return hipGetLastError();
}

hipError_t launch_append(int dtype, void* K, void* V, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                         const int32_t* seq_lens, const void* k_new, const void* v_new, int units, int n_kv_heads,
                         int max_ctx, hipStream_t st) {
  if (dtype == DT_F16)
    append_kernel<DT_F16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, kabsmax, seq_lens,
                                                (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx);
  else
    append_kernel<DT_BF16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, kabsmax, seq_lens,
                                                 (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx);
  return hipGetLastError();
}

}  // namespace fier
