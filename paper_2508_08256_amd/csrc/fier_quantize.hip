// 1-bit group quantizer of the key cache (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3)
// and the decode-stage append of Sec. 3.1.
//
// Group size 32 (the default; larger groups, g = 64 / 128 / 256, take quantize_long_kernel below):
// one wavefront owns one pair block (64 tokens = two groups of 32).  Lane l owns channels 2l and 2l+1:
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
#include "fier_quant_dev.h"

#pragma clang fp contract(off)

namespace fier {

// grid (ceil(n_pairs / 4), units), block 256: wave w of block x owns pair block 4x + w.
template <int DT>
__global__ __launch_bounds__(256) void quantize_kernel(const uint32_t* __restrict__ K, uint32_t* __restrict__ kbits,
                                                       uint32_t* __restrict__ kmeta, float* __restrict__ kabsmax,
                                                       const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                       int max_ctx, KvLayout lay) {
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
      const uint32_t* src = K + lay.rows_of(unit).row(t0) * (kD / 2) + lane;
#pragma unroll
      for (int t = 0; t < kG; ++t) rows[t] = src[(size_t)(t < ntok ? t : 0) * (kD / 2)];
      GroupCode gc;
      quantize_group<DT>(rows, ntok, lane, h * kG, mine, gc);
      meta0 = gc.meta_lo;
      meta1 = gc.meta_hi;
      amax0 = fmaxf(amax0, gc.amax_lo);
      amax1 = fmaxf(amax1, gc.amax_hi);
    }
    uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + 2 * P + h) * kD) + lane;
    *mdst = make_uint2(meta0, meta1);
  }
  reinterpret_cast<uint4*>(kbits)[(size_t)unit * max_ctx + P * kPair + lane] = mine;
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, amax0);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, amax1);
}

// Groups of g = 32 ns tokens, ns in {2, 4, 8}.  grid (ceil(n_groups / 4), units), block 256: wave w of block x owns
// group 4x + w.  The group's rows are read twice (min / max, then codes), 32 at a time; the second read hits L2.
template <int DT>
__global__ __launch_bounds__(256) void quantize_long_kernel(const uint32_t* __restrict__ K,
                                                            uint32_t* __restrict__ kbits,
                                                            uint32_t* __restrict__ kmeta, float* __restrict__ kabsmax,
                                                            const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                            int max_ctx, int ns, KvLayout lay) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int unit = blockIdx.y;
  const int g = kG * ns;
  const int Gi = blockIdx.x * 4 + wave;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int t0 = Gi * g;
  if (t0 >= L) return;
  const int ntok = L - t0 > g ? g : L - t0;
  const int n_groups = max_ctx / g;
  const uint32_t* src = K + lay.rows_of(unit).row(t0) * (kD / 2) + lane;
  auto row_at = [&](int t) { return src[(size_t)t * (kD / 2)]; };
  const GroupScale gs = long_group_scale<DT>(row_at, ntok);
  uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi) * kD) + lane;
  *mdst = make_uint2(gs.s0 | (gs.z0 << 16), gs.s1 | (gs.z1 << 16));
  for (int pb = 0; pb * kPair < ntok; ++pb) {
    uint4 mine = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c0 = pb * kPair + h * kG;
      int nt = ntok - c0;
      nt = nt > kG ? kG : nt;
      if (nt > 0) {
        uint32_t rows[kG];
#pragma unroll
        for (int t = 0; t < kG; ++t) rows[t] = row_at(c0 + t < ntok ? c0 + t : 0);
        uint32_t b0, b1;
        code_rows<DT>(rows, nt, gs, lane, h * kG, mine, b0, b1);
      }
    }
    reinterpret_cast<uint4*>(kbits)[(size_t)unit * max_ctx + t0 + pb * kPair + lane] = mine;
  }
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, fmaxf(fabsf(gs.zf0), fabsf(gs.zf0 + gs.sf0)));
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, fmaxf(fabsf(gs.zf1), fabsf(gs.zf1 + gs.sf1)));
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
                                                    const uint32_t* __restrict__ v_new, int n_kv_heads, int max_ctx,
                                                    int ns, KvLayout lay) {
  const int lane = threadIdx.x;
  const int unit = blockIdx.x;
  const int L = seq_lens[unit / n_kv_heads];
  if (L < 0 || L >= max_ctx) return;
  const uint32_t kn = k_new[(size_t)unit * (kD / 2) + lane];
  const uint32_t vn = v_new[(size_t)unit * (kD / 2) + lane];
  int t0, ntok;
  float amax_lo, amax_hi;
  if (ns == 1) {
    GroupCode gc;
    append_row<DT>(K, V, lay.rows_of(unit), kbits, kmeta, unit, L, max_ctx, kn, vn, lane, gc, t0, ntok);
    amax_lo = gc.amax_lo, amax_hi = gc.amax_hi;
  } else {
    const GroupScale gs = append_row_long<DT>(K, V, lay.rows_of(unit), kbits, kmeta, unit, L, max_ctx, ns, kn, vn, lane,
                                              t0, ntok,
                                              [](int, const uint4&, const GroupScale&) {});
    amax_lo = fmaxf(fabsf(gs.zf0), fabsf(gs.zf0 + gs.sf0));
    amax_hi = fmaxf(fabsf(gs.zf1), fabsf(gs.zf1 + gs.sf1));
  }
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, amax_lo);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, amax_hi);
}

hipError_t launch_quantize(int dtype, KvLayout lay, const void* K, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                           const int32_t* seq_lens, int units, int n_kv_heads, int max_ctx, int group_size,
                           hipStream_t st) {
  zero_absmax_kernel<<<(units * kD + 255) / 256, 256, 0, st>>>(kabsmax, units * kD);
  const int ns = group_size / kG;
  if (ns > 1) {
    dim3 grid_long((max_ctx / group_size + 3) / 4, units);
    if (dtype == DT_F16)
      quantize_long_kernel<DT_F16><<<grid_long, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens,
                                                             n_kv_heads, max_ctx, ns, lay);
    else
      quantize_long_kernel<DT_BF16><<<grid_long, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens,
                                                              n_kv_heads, max_ctx, ns, lay);
    return hipGetLastError();
  }
  dim3 grid((max_ctx / kPair + 3) / 4, units);
  if (dtype == DT_F16)
    quantize_kernel<DT_F16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, n_kv_heads,
                                                  max_ctx, lay);
  else
    quantize_kernel<DT_BF16><<<grid, 256, 0, st>>>((const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, n_kv_heads,
                                                   max_ctx, lay);
  return hipGetLastError();
}

hipError_t launch_append(int dtype, KvLayout lay, void* K, void* V, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                         const int32_t* seq_lens, const void* k_new, const void* v_new, int units, int n_kv_heads,
                         int max_ctx, int group_size, hipStream_t st) {
  const int ns = group_size / kG;
  if (dtype == DT_F16)
    append_kernel<DT_F16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, kabsmax, seq_lens,
                                                (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx,
                                                ns, lay);
  else
    append_kernel<DT_BF16><<<units, 64, 0, st>>>((uint32_t*)K, (uint32_t*)V, kbits, kmeta, kabsmax, seq_lens,
                                                 (const uint32_t*)k_new, (const uint32_t*)v_new, n_kv_heads, max_ctx,
                                                 ns, lay);
  return hipGetLastError();
}

}  // namespace fier
