// Approximate scores from the 1-bit key cache (Alg. 1 step 2):
//   score[j] = sum_c q_c * (z[G(j)][c] + bit[j][c] * s[G(j)][c]),  q = sum of the unit's query heads.
//
// The contraction over the 128 channels runs on the matrix cores as an int8 product
// (v_mfma_i32_16x16x64_i8), one wavefront per pair block (64 tokens = groups 2P and 2P+1) at a time:
//   * B operand = the codes.  A byte with a single bit k set IS the integer 2^k (bit 7: -128), so one v_and of a
//     code word with 0x01010101 << k yields four B elements: 8 vector ops expand 32 codes.  Lane (n, kq) of the
//     wavefront owns word kq of token n of a 16-token tile, which is exactly the B layout (k = 16 kq + 0..15);
//     the words arrive as one 16-byte load per token and are put into that order by four lane-row swaps;
//   * A operand = the weights.  w = q_c s_c (binary32 product), divided by its bit's power of two and turned
//     into a 31-bit fixed-point number relative to the largest |w| of its own group (the scale is a power of
//     two, found per group with a DPP max), then cut into four signed bytes: F = d0 + 2^8 d1 + 2^16 d2 + 2^24 d3.
//     The four digits are four rows of A.  The rows are built once per pair block by the lanes that hold the
//     group's (s, z) and reach the A layout through 1.3 KiB of LDS per wavefront;
//   * the digit rows are read back as two A operands, one with the digits in rows 0-3 / 8-11 and zeros elsewhere
//     for the first tile of each group, one with them in rows 4-7 / 12-15 for the second tile: both tiles of a
//     group accumulate into one 16x16 result that holds tile t in rows 4t..4t+3, the rows lane row t receives.
//     Lane l ends up with the four digit sums of token l of the block, recombines them in binary32 and adds
//     base[G] = sum_c q_c z[G][c];
//   * the integer accumulation is exact; the only rounding is the fixed-point step of the weights,
//     <= 2^(k-1) * 2^-30 * 2 max_c|w_c| per channel, about 4e-6 max|w| in the worst case over 128 channels.
//
// Channel bookkeeping.  Row r = lane / 16 works for group g = r / 2 and channel half h = r % 2; lane n of the row
// loads (s, z) of channels c = 64h + 4n + e, e = 0..3, as one 16-byte request.  Channel c sits in code word
// kq = h + 2(e & 1) at bit i = 2n + (e >> 1), i.e. byte y = i / 8, bit k = i % 8: MFMA j = k / 4, B register
// r = k % 4, contraction index K = 16 kq + 4r + y.
#include <type_traits>

#include "fier_dev.h"
#include "fier_kernels.h"
#include "fier_quant_dev.h"

namespace fier {

typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));


// LDS image of one wavefront's A operand: [j (K half)][group][digit][64 bytes], a zero row per j, padded so that
// the (group, j) sub-blocks start in different banks.
constexpr int kADigit = 64;
constexpr int kAGroup = 320;
constexpr int kAZeroRow = 576;
constexpr int kAPlane = 672;
constexpr int kAWave = 2 * kAPlane;
constexpr int kScoreMaxBpw = 13;  // pair blocks per wavefront at most (the launcher keeps to it)

__device__ __forceinline__ float wave_allsum(float x) {
  x = row_allsum(x);
  x += __shfl_xor(x, 16, 64);
  x += __shfl_xor(x, 32, 64);
  return x;
}

// value of the lane 16 away (rows 0 <-> 1, 2 <-> 3)
__device__ __forceinline__ float swap_rows(float x) {
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401f));  // bit mode: xor 16
}
// max over the 16 lanes of a row of non-negative floats, as unsigned integers (their bit patterns order alike)
template <int N>
__device__ __forceinline__ uint32_t row_ror_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + N, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t row_allmax_u32(uint32_t x) {
  x = max(x, row_ror_u32<8>(x));
  x = max(x, row_ror_u32<4>(x));
  x = max(x, row_ror_u32<2>(x));
  x = max(x, row_ror_u32<1>(x));
  return x;
}

// grid (units * (n_x [+ 1 if HIST])), n_x = ceil(max_ctx / (256 bpw)), block 256: scoring workgroup x of a unit
// owns 4 bpw consecutive pair blocks, wave w the blocks 4 bpw x + w, + 4, + 8, ...  The launcher picks bpw so that the whole grid is
// resident at once: the per-workgroup prologue (q, R) and epilogue (histogram flush, arrival) are then paid once.
//
// HIST (first kernel of the fused step): every score is also counted in an equal-width histogram of kSelBins
// bins over [-R, R], R = sum_c |q_c| * absmax_c >= |score| -- a bound known before any score exists, so that
// scoring and histogramming are one pass.  The workgroup's LDS histogram is added to the unit's histogram in
// memory with device atomics and the workgroup is done: nobody waits or counts arrivals here; the threshold
// kernel reads the merged histogram (and clears it for the next call).
// The extra workgroup of a unit performs the decode-stage append (Sec. 3.1) when k_new is given: one wavefront
// writes the new K/V rows, re-quantizes the group the row falls in and scores that group's tokens straight from
// its registers; the other workgroups leave those tokens alone.  The bound R uses the absmax of before the
// append (every workgroup must bin with the same R); the new group's contribution is handed to the last kernel
// of the step through `newmax`.  A score outside [-R, R] simply lands in the outermost bin.
template <int DT, int NREP, bool HIST, bool STREAM>
__global__ __launch_bounds__(256) void score_kernel(const uint4* kbits, const uint4* kmeta,
                                                    const float* __restrict__ kabsmax, const uint16_t* __restrict__ q,
                                                    const int32_t* __restrict__ seq_lens, int extra,
                                                    float* __restrict__ scores, UnitCtl* __restrict__ ctl,
                                                    uint32_t* __restrict__ ghist, const int32_t* __restrict__ budgets,
                                                    int max_budget, uint32_t* __restrict__ K, uint32_t* __restrict__ V,
                                                    const uint32_t* __restrict__ k_new,
                                                    const uint32_t* __restrict__ v_new, float* __restrict__ newmax,
                                                    int n_kv_heads, int max_ctx, int bpw, int gshift, int n_x, KvLayout lay) {
  __shared__ uint32_t lhist[HIST ? kSelBins : 1];
  __shared__ __attribute__((aligned(16))) unsigned char a_lds[4 * kAWave];
  // The workgroup's scores wait here and leave as one contiguous burst at the end: stores interleaved block by block
  // with the loads make the memory turn around between reading and writing all the time.
  __shared__ __attribute__((aligned(16))) float lscore[kScoreMaxBpw * 4 * kPair];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  // Workgroups are dispatched in the order of their index.  HIST: the first `units` workgroups are the appending
  // ones (their single wavefront has the longest chain of dependent loads: started last, it would end the kernel
  // late), then n_x scoring workgroups per unit, a unit's ranges next to each other.
  const int n_units = (int)gridDim.x / (n_x + (HIST ? 1 : 0));
  const bool append_wg = HIST && (int)blockIdx.x < n_units;
  const int wid = (int)blockIdx.x - (HIST ? n_units : 0);
  const int unit = append_wg ? (int)blockIdx.x : wid / n_x;
  const int range = append_wg ? -1 : wid - unit * n_x;
  const int b = unit / n_kv_heads;
  const uint16_t* qb = q + (size_t)unit * NREP * kD;
  // The appending wavefront's chain of dependent loads is the longest in the kernel: what it needs and what does
  // not depend on the sequence length (the new rows, its lanes' query values) leaves before anything else.
  uint32_t kn = 0, vn = 0, qpair[NREP];
#pragma unroll
  for (int r = 0; r < NREP; ++r) qpair[r] = 0;
  if (append_wg && wave == 0 && k_new != nullptr) {
    kn = k_new[(size_t)unit * (kD / 2) + lane];
    vn = v_new[(size_t)unit * (kD / 2) + lane];
#pragma unroll
    for (int r = 0; r < NREP; ++r) qpair[r] = reinterpret_cast<const uint32_t*>(qb + r * kD)[lane];
  }
  int Lold = seq_lens[b];
  Lold = Lold < 0 ? 0 : (Lold > max_ctx ? max_ctx : Lold);
  const bool app = HIST && k_new != nullptr && Lold < max_ctx;  // this unit receives a new row in this step
  int L = HIST ? Lold + (app ? 1 : 0) : Lold + extra;
  L = L > max_ctx ? max_ctx : L;
  const int gsize = kG << gshift;  // tokens per quantization group: 32, 64, 128 or 256
  const int tail_start = app ? (Lold / gsize) * gsize : L;  // tokens from here on are scored by the appending wave
  if (append_wg) {
    if (!app) return;
  } else {
    // range 0 of a unit always runs so that an empty unit still gets its control block written
    if (range * (4 * kPair) * bpw >= L && !(HIST && range == 0)) return;
  }
  // ... and the rows of the group the new token falls in as soon as the length is known (g = 32; the longer groups
  // read theirs in two passes inside append_row_long)
  uint32_t tail_rows[kG];
  int tail_t0 = 0, tail_ntok = 0;
  if (HIST && append_wg && wave == 0 && gshift == 0)
    append_load_rows<DT>(K, lay.rows_of(unit), Lold, kn, lane, tail_rows, tail_t0, tail_ntok);
  const int n_groups = max_ctx / gsize;
  const int row = lane >> 4, n = lane & 15;
  const int gsel = row >> 1;  // the group of the pair block whose (s, z) this row of lanes holds
  const int hsel = row & 1;   // the 64-channel half it holds
  FIER_PROF(0, HIST && unit == 0 && range == 3)
  if (HIST) { FIER_PROF_WG(0) }
  FIER_PROF(7, HIST && unit == 0 && append_wg)

  // ---- first block's loads go out before anything else (their addresses do not depend on q) ----------------
  const int P0 = range * (4 * bpw) + wave;  // this wave's blocks: P0, P0 + 4, ...
  const int lim = L < tail_start ? L : tail_start;  // tokens below this are scored by the scoring workgroups
  const bool scoring = !append_wg && P0 * kPair < lim;
  const uint32_t* __restrict__ bits_u = reinterpret_cast<const uint32_t*>(kbits) + (size_t)unit * max_ctx * 4;
  const uint4* __restrict__ meta_u = kmeta + (size_t)unit * n_groups * (kD / 4);
  // lane l loads the whole 16-byte code word of token l of the block (one contiguous 1 KiB request per wavefront);
  // the lane's (s, z) quad of block P is at meta_u[((2 P + gsel) >> gshift) * 32 + 16 hsel + n]: half-block
  // 2 P + gsel (32 tokens) lies in group (2 P + gsel) >> gshift
  const uint4* const pb = reinterpret_cast<const uint4*>(bits_u) + ((size_t)P0 * kPair + lane);
  const uint4* const pm = meta_u + ((size_t)((2 * P0 + gsel) >> gshift) * 32 + 16 * hsel + n);
  const int pm_step = 256 >> gshift;  // uint4 per block step: a wave's next block is 4 blocks = 8 half-blocks on
  // blocks of this wave that hold tokens to score: P0, P0 + 4, ... below ceil(lim / 64), at most bpw; only the
  // last of them can be a partial one
  int nb = scoring ? ((lim + kPair - 1) / kPair - P0 + 3) / 4 : 0;
  nb = nb > bpw ? bpw : nb;
  // block P0 + 4 i of this wave; past the wave's last block the last one is fetched again (unconditional loads
  // keep the count of outstanding requests the same on every path)
  auto fetch = [&](uint32_t (&w)[4], uint4& m, int i) {
    i = i < nb ? i : nb - 1;
    // STREAM: the codes and metadata are read once per step and, from a size on, are better kept out of the caches
    // (see the launcher)
    const uint4 v = STREAM ? load_stream(pb + (size_t)i * (4 * kPair)) : pb[(size_t)i * (4 * kPair)];
    w[0] = v.x;
    w[1] = v.y;
    w[2] = v.z;
    w[3] = v.w;
    m = STREAM ? load_stream(pm + (size_t)i * pm_step) : pm[(size_t)i * pm_step];
  };
  uint32_t w_cur[4] = {0, 0, 0, 0};
  uint4 m_cur = make_uint4(0, 0, 0, 0);
  if (scoring) fetch(w_cur, m_cur, 0);

  // ---- the lane's 4 query channels c = 64 hsel + 4 n + e, summed over the query heads of this kv head ------
  float qs[4];
  float R = 0.f, hscale = 0.f;
  {
#pragma unroll
    for (int e = 0; e < 4; ++e) qs[e] = 0.f;
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
      const uint2 qq = *reinterpret_cast<const uint2*>(qb + r * kD + 64 * hsel + 4 * n);
      qs[0] += lo16f<DT>(qq.x);
      qs[1] += hi16f<DT>(qq.x);
      qs[2] += lo16f<DT>(qq.y);
      qs[3] += hi16f<DT>(qq.y);
    }
    if (HIST) {
      const float4 am = *reinterpret_cast<const float4*>(kabsmax + (size_t)unit * kD + 64 * hsel + 4 * n);
      float rpart = fabsf(qs[0]) * am.x;
      rpart += fabsf(qs[1]) * am.y;
      rpart += fabsf(qs[2]) * am.z;
      rpart += fabsf(qs[3]) * am.w;
      rpart = row_allsum(rpart);   // this half of the channels
      rpart += swap_rows(rpart);   // both halves
      // lane 0's sum is taken so that R is bit-identical in every lane, wave and workgroup (the binning must be
      // the same function everywhere)
      R = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(rpart)));
      hscale = sel_scale(R, kSelBins);
      for (int i = tid; i < kSelBins; i += 256) lhist[i] = 0;
      __syncthreads();
    }
  }

  FIER_PROF(1, HIST && unit == 0 && range == 3)
  if (append_wg) {
    if constexpr (HIST) {
      if (wave == 0 && gshift == 0) {  // lane = channel pair (2 lane, 2 lane + 1)
        GroupCode gc;
        const int t0 = tail_t0, ntok = tail_ntok;
        uint4 mine;  // lane t < 32: the code word of token t0 + t
        append_finish<DT>(K, V, lay.rows_of(unit), const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kbits)),
                          const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kmeta)), unit, Lold, max_ctx, kn, vn,
                          lane, tail_rows, t0, ntok, gc, mine);
        newmax[(size_t)unit * kD + 2 * lane] = gc.amax_lo;
        newmax[(size_t)unit * kD + 2 * lane + 1] = gc.amax_hi;
        float q0 = 0.f, q1 = 0.f;
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
          q0 += lo16f<DT>(qpair[r]);
          q1 += hi16f<DT>(qpair[r]);
        }
        // lane = token: the 128 weights q_c s_c go through LDS in the order of the code word's bits (channel 2 lane
        // is bit lane & 31 of word lane >> 5, channel 2 lane + 1 of word 2 + (lane >> 5)); every lane then adds up
        // the weights of its own token's set bits -- one wavefront-wide sum (the base) instead of one per token
        float* wl = reinterpret_cast<float*>(a_lds);  // 128 floats; this workgroup scores nothing else
        wl[lane] = q0 * gc.s_lo;
        wl[64 + lane] = q1 * gc.s_hi;
        const float base = wave_allsum(q0 * gc.z_lo + q1 * gc.z_hi);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t wd[4] = {mine.x, mine.y, mine.z, mine.w};
        float acc = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int i = 0; i < 32; i += 4) {
            const float4 w4 = *reinterpret_cast<const float4*>(wl + 32 * d + i);
            acc += (wd[d] >> i & 1u) ? w4.x : 0.f;
            acc += (wd[d] >> (i + 1) & 1u) ? w4.y : 0.f;
            acc += (wd[d] >> (i + 2) & 1u) ? w4.z : 0.f;
            acc += (wd[d] >> (i + 3) & 1u) ? w4.w : 0.f;
          }
        if (lane < ntok) {
          const float sc = acc + base;
          scores[(size_t)unit * max_ctx + t0 + lane] = sc;
          atomicAdd(&lhist[sel_bin(sc, R, hscale, kSelBins)], 1u);
        }
      } else if (wave == 0) {
        // Groups of 64, 128 or 256 tokens: the tail group is re-derived 32 rows at a time; each of its pair blocks
        // is scored as soon as its code words exist, lane = token, the 128 weights q_c s_c read from LDS in the
        // order of the code word's bits (bit i of word d is channel 64 (d & 1) + 2 i + (d >> 1)).
        float* wl = reinterpret_cast<float*>(a_lds);  // 128 floats; this workgroup scores nothing else
        float q0 = 0.f, q1 = 0.f;
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
          q0 += lo16f<DT>(qpair[r]);
          q1 += hi16f<DT>(qpair[r]);
        }
        int t0, ntok;
        float base = 0.f;
        bool have_w = false;
        const GroupScale gs = append_row_long<DT>(
            K, V, lay.rows_of(unit), const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kbits)),
            const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kmeta)), unit, Lold, max_ctx, 1 << gshift, kn, vn, lane,
            t0, ntok, [&](int pb, const uint4& mine, const GroupScale& g) {
              if (!have_w) {
                have_w = true;
                // channel 2 lane is bit (lane & 31) of word lane >> 5, channel 2 lane + 1 of word 2 + (lane >> 5)
                wl[lane] = q0 * g.sf0;
                wl[64 + lane] = q1 * g.sf1;
                base = wave_allsum(q0 * g.zf0 + q1 * g.zf1);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
              }
              const uint32_t wd[4] = {mine.x, mine.y, mine.z, mine.w};
              float acc = 0.f;
#pragma unroll
              for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int i = 0; i < 32; i += 4) {
                  const float4 w4 = *reinterpret_cast<const float4*>(wl + 32 * d + i);
                  acc += (wd[d] >> i & 1u) ? w4.x : 0.f;
                  acc += (wd[d] >> (i + 1) & 1u) ? w4.y : 0.f;
                  acc += (wd[d] >> (i + 2) & 1u) ? w4.z : 0.f;
                  acc += (wd[d] >> (i + 3) & 1u) ? w4.w : 0.f;
                }
              const int tok = pb * kPair + lane;  // within the group
              if (tok < ntok) {
                const float sc = acc + base;
                scores[(size_t)unit * max_ctx + t0 + tok] = sc;
                atomicAdd(&lhist[sel_bin(sc, R, hscale, kSelBins)], 1u);
              }
            });
        newmax[(size_t)unit * kD + 2 * lane] = fmaxf(fabsf(gs.zf0), fabsf(gs.zf0 + gs.sf0));
        newmax[(size_t)unit * kD + 2 * lane + 1] = fmaxf(fabsf(gs.zf1), fabsf(gs.zf1 + gs.sf1));
      }
    }
  }

  if (scoring) {
    // per-lane constants of the weight rows
    float qk[4];   // q_c divided by the integer its code bit stands for in B
    int a_wr[4];   // LDS byte offset of digit 0 of channel e
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int kq_c = hsel + 2 * (e & 1);
      const int i_c = 2 * n + (e >> 1);
      const int y = i_c >> 3, k = i_c & 7;
      // 2^-k, negative for k = 7 (a byte with only bit 7 set is -128)
      const float inv_bit = __uint_as_float(((uint32_t)(127 - k) << 23) | (k == 7 ? 0x80000000u : 0u));
      qk[e] = qs[e] * inv_bit;
      a_wr[e] = wave * kAWave + (k >> 2) * kAPlane + gsel * kAGroup + 16 * kq_c + 4 * (k & 3) + y;
    }
    // Two A operands.  "Even" serves the first tile of each group and carries the digits of the first group in
    // rows 0-3, of the second in rows 8-11; "odd" serves the second tiles with the same digits in rows 4-7 and
    // 12-15; all other rows read the zero row.  The two tiles of a group then accumulate into one 16x16 result
    // that holds tile t in rows 4t..4t+3, the rows lane row t receives.
    if (lane < 32) *reinterpret_cast<uint32_t*>(a_lds + wave * kAWave + (lane >> 4) * kAPlane + kAZeroRow + 4 * n) = 0u;
    const int a_real = (n >> 3) * kAGroup + (n & 3) * kADigit;
    const int a_even = wave * kAWave + ((n & 4) ? kAZeroRow : a_real) + 16 * row;
    const int a_odd = wave * kAWave + ((n & 4) ? a_real : kAZeroRow) + 16 * row;

    // full_tag: every token of the block is below `lim`.  The store and the count are then unmasked, so the number
    // of memory operations in flight is the same on every path and the wait for the next block's loads can leave
    // this block's store outstanding -- with a masked store the compiler has to wait for everything, and the
    // store's acknowledgement (it is the last operation issued) lands on the critical path of every iteration.
    auto score_block = [&](auto full_tag, int it) {
      constexpr bool FULL = decltype(full_tag)::value;
      const int P = P0 + 4 * it;
      // The B layout wants, in lane (row r, n), word r of the tokens 16 t + n, t = 0..3; the load left word d of
      // token 16 r + n in register d: a 4x4 transpose between register index and lane row, two swap stages.
      {
        const u32x2_t a = __builtin_amdgcn_permlane32_swap(w_cur[0], w_cur[2], false, false);
        const u32x2_t b = __builtin_amdgcn_permlane32_swap(w_cur[1], w_cur[3], false, false);
        const u32x2_t c = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
        const u32x2_t d = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
        w_cur[0] = c[0];
        w_cur[1] = c[1];
        w_cur[2] = d[0];
        w_cur[3] = d[1];
      }

      // ---- this row's weights -> fixed point relative to the group's largest -> digit rows in LDS ----------
      const uint32_t mw[4] = {m_cur.x, m_cur.y, m_cur.z, m_cur.w};
      float wv[4];
      float basep = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        wv[e] = qk[e] * lo16f<DT>(mw[e]);
        basep += qs[e] * hi16f<DT>(mw[e]);
      }
      uint32_t mx = __float_as_uint(fmaxf(fmaxf(fabsf(wv[0]), fabsf(wv[1])), fmaxf(fabsf(wv[2]), fabsf(wv[3]))));
      mx = row_allmax_u32(mx);
      mx = max(mx, (uint32_t)__builtin_amdgcn_ds_swizzle((int)mx, 0x401f));  // over all 128 channels of the group
      // max|w| < 2^(ex - 126), ex its biased exponent: scale = 2^(156 - ex) keeps |w * scale| < 2^30
      uint32_t exb = mx & 0x7f800000u;
      exb = exb < (29u << 23) ? (29u << 23) : exb;
      const float scale = __uint_as_float(0x8d800000u - exb);      // (283 - ex) << 23
      const float inv_scale = __uint_as_float(exb - (29u << 23));  // 2^(ex - 156); 0 when the group carries nothing
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int F = (int)rintf(wv[e] * scale);
        // signed digits: the bytes of (F + 0x808080) ^ 0x808080, the top one as it is
        const uint32_t X = ((uint32_t)F + 0x00808080u) ^ 0x00808080u;
        unsigned char* dst = a_lds + a_wr[e];
        dst[0] = (unsigned char)X;
        dst[kADigit] = (unsigned char)(X >> 8);
        dst[2 * kADigit] = (unsigned char)(X >> 16);
        dst[3 * kADigit] = (unsigned char)(X >> 24);
      }
      float base = row_allsum(basep);
      base += swap_rows(base);  // every lane of rows 2g, 2g + 1: base of group g
      // the writes above come from other lanes of this same wavefront: LDS operations of a wavefront complete
      // in order, the fences keep the compiler from moving the reads above them
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // ---- 4 tiles x 2 K-halves ----------------------------------------------------------------------------
      const i32x4_t ae0 = *reinterpret_cast<const i32x4_t*>(a_lds + a_even);
      const i32x4_t ae1 = *reinterpret_cast<const i32x4_t*>(a_lds + a_even + kAPlane);
      const i32x4_t ao0 = *reinterpret_cast<const i32x4_t*>(a_lds + a_odd);
      const i32x4_t ao1 = *reinterpret_cast<const i32x4_t*>(a_lds + a_odd + kAPlane);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // reads done before the next block's writes
      i32x4_t acc[2];
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        i32x4_t b[2][2];  // [tile of the group][K half]
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            b[u][0][r] = (int)(w_cur[2 * g + u] & (0x01010101u << r));
            b[u][1][r] = (int)(w_cur[2 * g + u] & (0x01010101u << (4 + r)));
          }
        acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ae0, b[0][0], i32x4_t{0, 0, 0, 0}, 0, 0, 0);
        acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ae1, b[0][1], acc[g], 0, 0, 0);
        acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ao0, b[1][0], acc[g], 0, 0, 0);
        acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ao1, b[1][1], acc[g], 0, 0, 0);
      }
      // lane l = 16 row + n is token l of the block: its digit sums are registers 0..3 of its group's result
      const i32x4_t dg = gsel ? acc[1] : acc[0];
      float f = (float)dg[0];
      f = fmaf((float)dg[1], 256.0f, f);
      f = fmaf((float)dg[2], 65536.0f, f);
      f = fmaf((float)dg[3], 16777216.0f, f);
      const float sc = fmaf(f, inv_scale, base);
      const int tok = P * kPair + lane;
      lscore[(wave + 4 * it) * kPair + lane] = sc;
      if (HIST && (FULL || tok < lim)) atomicAdd(&lhist[sel_bin(sc, R, hscale, kSelBins)], 1u);
    };
    for (int it = 0; it + 1 < nb; ++it) {
      uint32_t w_nxt[4];
      uint4 m_nxt;
      fetch(w_nxt, m_nxt, it + 1);  // the next block is on its way while this one is scored
      score_block(std::true_type(), it);
#pragma unroll
      for (int t = 0; t < 4; ++t) w_cur[t] = w_nxt[t];
      m_cur = m_nxt;
    }
    score_block(std::false_type(), nb - 1);  // the wave's last block may be a partial one
  }

  // ---- the workgroup's scores: tokens [tok_wg, min(tok_wg + 256 bpw, lim)) in one go ------------------------------
  if (!append_wg) {
    __syncthreads();
    const int tok_wg = range * (4 * kPair) * bpw;
    int n_wg = lim - tok_wg;
    n_wg = n_wg > 4 * kPair * bpw ? 4 * kPair * bpw : n_wg;
    float* __restrict__ dst = scores + (size_t)unit * max_ctx + tok_wg;  // tok_wg is a multiple of 256: 16-byte aligned
    for (int i = 4 * tid; i < n_wg; i += 4 * 256) {
      const float4 v4 = *reinterpret_cast<const float4*>(lscore + i);
      if (i + 3 < n_wg) {
        if constexpr (HIST) {
          // the step's second kernel reads them once, after this kernel has ended: stored with the streaming hint
          // (0.5 us per step at the 64k and 128k shapes, nothing at the others)
          typedef float f4_t __attribute__((ext_vector_type(4)));
          __builtin_nontemporal_store(f4_t{v4.x, v4.y, v4.z, v4.w}, reinterpret_cast<f4_t*>(dst + i));
        } else {
          *reinterpret_cast<float4*>(dst + i) = v4;
        }
      } else {
        dst[i] = v4.x;
        if (i + 1 < n_wg) dst[i + 1] = v4.y;
        if (i + 2 < n_wg) dst[i + 2] = v4.z;
      }
    }
  }
  FIER_PROF(2, HIST && unit == 0 && range == 3)
  FIER_PROF(8, HIST && unit == 0 && append_wg)
  if constexpr (HIST) {
    __syncthreads();
    uint32_t* __restrict__ gh = ghist + (size_t)unit * kSelBins;
    for (int i = tid; i < kSelBins; i += 256) {
      const uint32_t c = lhist[i];
      if (c) atomicAdd(&gh[i], c);
    }
    // the bound the scores were binned with, for the kernels that follow (range 0 of a unit always runs)
    if (range == 0 && tid == 0) {
      UnitCtl* c = &ctl[unit];
      c->R = R;
      c->scale = hscale;
    }
    FIER_PROF(3, unit == 0 && range == 3)
    FIER_PROF_WG(1)
  }
}

template <int DT, bool HIST>
static hipError_t launch_score_dt(KvLayout lay, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                                  const void* q, const int32_t* seq_lens, int extra, float* scores,
                                  const StepBuffers* sb, const int32_t* budgets, int max_budget, void* K, void* V,
                                  const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                                  int group_size, hipStream_t st) {
  const int gshift = group_size == 256 ? 3 : group_size == 128 ? 2 : group_size == 64 ? 1 : 0;
  // Blocks per wavefront.  The smallest that lets every workgroup be resident at once (256 CUs; the registers
  // allow 5 workgroups per CU for the fused kernel -- 4 with 8 query heads per kv head --, 8 for the score-only
  // one), at least 4: prologue (q, R) and epilogue (histogram flush) are then paid once.  Beyond 12 the grid is cut into several rounds of shorter
  // workgroups instead: a workgroup's lifetime bounds the ragged end of the kernel, and in a batch of unequal
  // contexts (the host cannot see the lengths) the short units' workgroups exit at once and the dispatcher
  // backfills the machine with the long units' -- with one round, a few long units would stream alone at one
  // block in flight per wavefront.  Strides of a power of two between the workgroups' streams are avoided (they
  // collide in the memory channels: measured 8 vs 7 or 9, 16 vs 13).
  const int n_blocks = (max_ctx + kPair - 1) / kPair;
  const int wg_slots = HIST ? 256 * 5 - units : 256 * 8;
  const int per_unit = wg_slots / units > 0 ? wg_slots / units : 1;
  int bpw = (n_blocks + 4 * per_unit - 1) / (4 * per_unit);
  bpw = bpw < 4 ? 4 : bpw;
  const int rounds = (bpw + 11) / 12;
  bpw = (bpw + rounds - 1) / rounds;
  if (bpw >= 8 && (bpw & (bpw - 1)) == 0) ++bpw;
  if (bpw > kScoreMaxBpw) return hipErrorInvalidValue;  // cannot happen: at most 12, + 1
  const int n_x = (n_blocks + 4 * bpw - 1) / (4 * bpw);  // scoring workgroups per unit
  dim3 grid((unsigned)units * (unsigned)(n_x + (HIST ? 1 : 0)));
  // Streaming hint on the loads of the codes and their metadata (read once per step).  Measured with the step
  // rotating over 12 layer caches, this kernel alone, us without / with it: 32 units x 128k 34.4 / 30.6, 32 x 64k
  // 19.2 / 16.5, the ragged 128-unit batch 34.5 / 31.5 (whole steps: 62.2 / 61.5, 32.6 / 31.9, 102.3 / 100.7);
  // shapes of 32 units x 32k and below lost 0.2-0.4 us per step with it.  Hence from 64 MB per launch.
  const bool stream = (long)units * max_ctx * 32 >= (64L << 20);
#define FIER_SCORE_ARGS                                                                                            \
  (const uint4*)kbits, (const uint4*)kmeta, kabsmax, (const uint16_t*)q, seq_lens, extra, scores,                  \
      sb ? sb->ctl : nullptr, sb ? sb->hist : nullptr, budgets, max_budget, (uint32_t*)K, (uint32_t*)V,            \
      (const uint32_t*)k_new, (const uint32_t*)v_new, sb ? sb->newmax : nullptr, n_kv_heads, max_ctx, bpw, gshift, \
      n_x, lay
#define FIER_SCORE_CASE(R)                                                                                         \
  case R:                                                                                                          \
    if (stream)                                                                                                    \
      score_kernel<DT, R, HIST, true><<<grid, 256, 0, st>>>(FIER_SCORE_ARGS);                                      \
    else                                                                                                           \
      score_kernel<DT, R, HIST, false><<<grid, 256, 0, st>>>(FIER_SCORE_ARGS);                                     \
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
#undef FIER_SCORE_ARGS
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
