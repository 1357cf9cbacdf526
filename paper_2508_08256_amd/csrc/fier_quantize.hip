// 1-bit group quantizer of the key cache (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3)
// and the decode-stage append of Sec. 3.1.
//
// Group size 32 (the default; the larger groups g = 64 / 128 / 256 differ in how min / max are combined):
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

typedef short short2_t __attribute__((ext_vector_type(2)));

// Both 16-bit floats of a word as signed integers that order like the floats (sign-magnitude -> two's
// complement; the map is its own inverse).  Minimum and maximum of finite values can then be taken two channels
// at a time with packed integer instructions, for fp16 and bf16 alike; -0 sorts below +0, which the
// canonicalisation of zeros in group_scale makes immaterial.
__device__ __forceinline__ short2_t order_keys(uint32_t pair) {
  const short2_t v = __builtin_bit_cast(short2_t, pair);
  return v ^ ((v >> 15) & (short)0x7fff);
}

// Whole groups.  grid (ceil(n_pairs / (4 bpw)), units), block 256: wave w of workgroup x owns the pair blocks
// 4 bpw x + w, + 4, + 8, ...; NS = group size / 32.  The 64 rows of a pair block sit in registers (one dword per
// row and lane, two halves of 32).  As soon as a half has been coded, its registers receive the same half of the
// wave's next block, so that 8 KiB per wavefront are in flight while the other half is worked on.
//   NS = 1: the two halves are two groups.   NS = 2: the pair block is one group.
//   NS = 4, 8: a group spans the pair blocks of 2 / 4 neighbouring wavefronts, which exchange their minima and
//   maxima through LDS (one barrier per block): every row is still read exactly once.
// A unit's last, partial group is left to the tail kernels.
template <int DT, int NS>
__global__ __launch_bounds__(256) void quantize_kernel(const uint32_t* __restrict__ K, uint32_t* __restrict__ kbits,
                                                       uint32_t* __restrict__ kmeta, float* __restrict__ kabsmax,
                                                       const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                       int max_ctx, int bpw, KvLayout lay) {
  constexpr int kWavesPerGroup = NS >= 4 ? NS / 2 : 1;
  __shared__ uint2 xch[2][4][64];  // [iteration parity][wavefront][lane]: packed (min, max) keys, NS >= 4 only
  const int lane = threadIdx.x & 63;
  // the wavefront's number as a scalar: everything derived from it (addresses, branches) is then uniform for the
  // compiler too
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int unit = blockIdx.y;
  const int base = blockIdx.x * (4 * bpw);
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  // pair blocks that consist of whole groups
  const int n_full = NS == 1 ? L / kPair : (L / (kG * NS)) * (NS / 2);
  if (base >= n_full) return;
  const int n_groups = max_ctx / (kG * NS);
  const KvRows kv = lay.rows_of(unit);
  auto load_half = [&](uint32_t (&rows)[kG], int P, int h) {
    const uint32_t* src = K + kv.row(P * kPair + h * kG) * (kD / 2) + lane;
#pragma unroll
    for (int t = 0; t < kG; ++t) rows[t] = load_stream(src + t * (kD / 2));
  };
  auto minmax_keys = [&](const uint32_t (&rows)[kG], short2_t& mn, short2_t& mx) {
    mn = mx = order_keys(rows[0]);
#pragma unroll
    for (int t = 1; t < kG; ++t) {
      const short2_t k = order_keys(rows[t]);
      mn = __builtin_elementwise_min(mn, k);
      mx = __builtin_elementwise_max(mx, k);
    }
  };
  auto scale_of = [&](short2_t mn, short2_t mx) {
    const uint32_t mnw = __builtin_bit_cast(uint32_t, order_keys(__builtin_bit_cast(uint32_t, mn)));
    const uint32_t mxw = __builtin_bit_cast(uint32_t, order_keys(__builtin_bit_cast(uint32_t, mx)));
    MinMax m;
    m.mn0 = lo16f<DT>(mnw), m.mn1 = hi16f<DT>(mnw);
    m.mx0 = lo16f<DT>(mxw), m.mx1 = hi16f<DT>(mxw);
    return group_scale<DT>(m);
  };
  float amax0 = 0.f, amax1 = 0.f;
  auto store_meta = [&](int group, const GroupScale& g) {
    uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + group) * kD) + lane;
    *mdst = make_uint2(g.s0 | (g.z0 << 16), g.s1 | (g.z1 << 16));
    amax0 = fmaxf(amax0, fmaxf(fabsf(g.zf0), fabsf(g.zf0 + g.sf0)));
    amax1 = fmaxf(amax1, fmaxf(fabsf(g.zf1), fabsf(g.zf1 + g.sf1)));
  };
  uint32_t ra[kG], rb[kG];
  if (base + wave < n_full) {
    load_half(ra, base + wave, 0);
    load_half(rb, base + wave, 1);
  }
  for (int i = 0; i < bpw; ++i) {
    if (base + 4 * i >= n_full) break;  // the same for the whole workgroup
    const int P = base + 4 * i + wave;
    const bool active = P < n_full;  // the wavefronts of one group are active together
    const bool more = i + 1 < bpw && P + 4 < n_full;
    short2_t mn_a, mx_a, mn_b, mx_b;
    if (active) {
      minmax_keys(ra, mn_a, mx_a);
      minmax_keys(rb, mn_b, mx_b);
      if constexpr (NS >= 2) {
        mn_a = __builtin_elementwise_min(mn_a, mn_b);
        mx_a = __builtin_elementwise_max(mx_a, mx_b);
      }
    }
    if constexpr (NS >= 4) {
      if (active)
        xch[i & 1][wave][lane] = make_uint2(__builtin_bit_cast(uint32_t, mn_a), __builtin_bit_cast(uint32_t, mx_a));
      __syncthreads();  // the buffer of the other parity is rewritten only after the next barrier
      if (active) {
        const int first = wave & ~(kWavesPerGroup - 1);
#pragma unroll
        for (int k = 1; k < kWavesPerGroup; ++k) {
          const uint2 o = xch[i & 1][first + ((wave + k) & (kWavesPerGroup - 1))][lane];
          mn_a = __builtin_elementwise_min(mn_a, __builtin_bit_cast(short2_t, o.x));
          mx_a = __builtin_elementwise_max(mx_a, __builtin_bit_cast(short2_t, o.y));
        }
      }
    }
    if (!active) continue;
    const GroupScale ga = scale_of(mn_a, mx_a);
    const GroupScale gb = NS == 1 ? scale_of(mn_b, mx_b) : ga;
    uint4 mine = make_uint4(0, 0, 0, 0);
    uint32_t b0, b1;
    code_rows<DT, true>(ra, kG, ga, lane, 0, mine, b0, b1);
    if (more) load_half(ra, P + 4, 0);
    code_rows<DT, true>(rb, kG, gb, lane, kG, mine, b0, b1);
    if (more) load_half(rb, P + 4, 1);
    reinterpret_cast<uint4*>(kbits)[(size_t)unit * max_ctx + P * kPair + lane] = mine;
    if constexpr (NS == 1) {
      store_meta(2 * P, ga);
      store_meta(2 * P + 1, gb);
    } else if ((P & (kWavesPerGroup - 1)) == 0) {  // the group's first wavefront
      store_meta(P / (NS / 2), ga);
    }
  }
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane, amax0);
  raise_absmax(kabsmax + (size_t)unit * kD + 2 * lane + 1, amax1);
}

// grid (units), block 64, g = 32: the unit's last pair block when it is partial (1 to 63 tokens present).
template <int DT>
__global__ __launch_bounds__(64) void quantize_tail_kernel(const uint32_t* __restrict__ K,
                                                           uint32_t* __restrict__ kbits,
                                                           uint32_t* __restrict__ kmeta, float* __restrict__ kabsmax,
                                                           const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                           int max_ctx, KvLayout lay) {
  const int lane = threadIdx.x;
  const int unit = blockIdx.x;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int P = L / kPair;
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

// grid (units), block 64, g = 32 ns with ns in {2, 4, 8}: the unit's last group when it is partial.  Its rows are
// read twice (min / max, then codes), 32 at a time.
template <int DT>
__global__ __launch_bounds__(64) void quantize_long_tail_kernel(const uint32_t* __restrict__ K,
                                                                uint32_t* __restrict__ kbits,
                                                                uint32_t* __restrict__ kmeta,
                                                                float* __restrict__ kabsmax,
                                                                const int32_t* __restrict__ seq_lens, int n_kv_heads,
                                                                int max_ctx, int ns, KvLayout lay) {
  const int lane = threadIdx.x;
  const int unit = blockIdx.x;
  const int g = kG * ns;
  int L = seq_lens[unit / n_kv_heads];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int Gi = L / g;
  const int t0 = Gi * g;
  if (t0 >= L) return;
  const int ntok = L - t0;
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
    uint4 mine;
    append_row<DT>(K, V, lay.rows_of(unit), kbits, kmeta, unit, L, max_ctx, kn, vn, lane, gc, t0, ntok, mine);
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

template <int DT>
static void launch_quantize_dt(KvLayout lay, const uint32_t* K, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                               const int32_t* seq_lens, int units, int n_kv_heads, int max_ctx, int ns, int bpw,
                               dim3 grid, hipStream_t st) {
#define FIER_Q_ARGS K, kbits, kmeta, kabsmax, seq_lens, n_kv_heads, max_ctx
  switch (ns) {
    case 1:
      quantize_kernel<DT, 1><<<grid, 256, 0, st>>>(FIER_Q_ARGS, bpw, lay);
      quantize_tail_kernel<DT><<<units, 64, 0, st>>>(FIER_Q_ARGS, lay);
      return;
    case 2: quantize_kernel<DT, 2><<<grid, 256, 0, st>>>(FIER_Q_ARGS, bpw, lay); break;
    case 4: quantize_kernel<DT, 4><<<grid, 256, 0, st>>>(FIER_Q_ARGS, bpw, lay); break;
    default: quantize_kernel<DT, 8><<<grid, 256, 0, st>>>(FIER_Q_ARGS, bpw, lay); break;
  }
  quantize_long_tail_kernel<DT><<<units, 64, 0, st>>>(FIER_Q_ARGS, ns, lay);
#undef FIER_Q_ARGS
}

hipError_t launch_quantize(int dtype, KvLayout lay, const void* K, uint32_t* kbits, uint32_t* kmeta, float* kabsmax,
                           const int32_t* seq_lens, int units, int n_kv_heads, int max_ctx, int group_size,
                           hipStream_t st) {
  zero_absmax_kernel<<<(units * kD + 255) / 256, 256, 0, st>>>(kabsmax, units * kD);
  const int ns = group_size / kG;
  // Pair blocks per wavefront: as many as make the grid about one resident round (256 CUs x 4 workgroups), at
  // most 12 (longer grids run in several rounds, see the score kernel's launcher for the reasons), and no power of
  // two from 4 on: such strides between the concurrently streaming workgroups collide in the memory channels
  // (config-2 shape: 93 / 82 / 105 / 86 us at 4 / 6 / 8 / 12).  One block per wavefront is 3 x slower: launch and
  // the per-wavefront update of the unit's absmax dominate.
  const int n_pairs = max_ctx / kPair;
  int bpw = (int)(((long)n_pairs * units + 4L * 1024 - 1) / (4L * 1024));
  const int rounds = (bpw + 11) / 12;
  bpw = (bpw + rounds - 1) / rounds;
  if (bpw >= 4 && (bpw & (bpw - 1)) == 0) ++bpw;
  // Nine blocks per wavefront wherever that still leaves a workgroup per CU: measured best at every large shape
  // (config-2 shape, us: 88 at 5, 86 at 7, 78 at 9, 81 at 10, 85 at 11, 82 at 17; the 128k shape gets 9 from the
  // rule above anyway).  The differences between neighbouring values are strides between the concurrently streaming
  // workgroups (bpw x 64 KiB) meeting the memory channels differently.
  if (bpw < 9 && (long)n_pairs * units >= 4L * 9 * 256) bpw = 9;
  dim3 grid((n_pairs + 4 * bpw - 1) / (4 * bpw), units);
  if (dtype == DT_F16)
    launch_quantize_dt<DT_F16>(lay, (const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, units, n_kv_heads, max_ctx, ns,
                               bpw, grid, st);
  else
    launch_quantize_dt<DT_BF16>(lay, (const uint32_t*)K, kbits, kmeta, kabsmax, seq_lens, units, n_kv_heads, max_ctx,
                                ns, bpw, grid, st);
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
