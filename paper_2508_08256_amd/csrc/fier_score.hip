// Approximate scores from the 1-bit key cache (Alg. 1 step 2):
//   score[j] = sum_c q_c * (z[G(j)][c] + bit[j][c] * s[G(j)][c]),  q = sum of the unit's query heads.
//
// Lane = token.  One wavefront owns one pair block (64 tokens = groups 2P and 2P+1) at a time:
//   * each lane loads the 16-byte code word of its own token (one coalesced 1 KiB request per block);
//   * the per-group weights w[c] = q_c * s[G][c] differ between the two halves of the wavefront.  They
//     stay distributed: each row of 16 lanes holds all 128 weights of its own group in 8 registers
//     (lane n of the row holds 8 channels), and a DPP row broadcast inside the multiply-add hands weight
//     (m, n) to the 16 lanes of the row.  No LDS and no replication through memory;
//   * "bit ? w : 0" costs no select: a code word ANDed with a single-bit mask in the exponent field of a
//     binary32 IS the number 2^k or 0 (bit 30 -> 2, 29 -> 2^-63, 28 -> 2^-95, 27 -> 2^-111).  The weight
//     register carries the inverse power of two (folded into q once per kernel), so one v_and and one
//     v_fmac with a DPP source accumulate bit * w exactly.  Eight rotations of each code word bring every
//     bit to one of the four usable positions: 2 + 7/32 vector ops per (token, channel);
//   * q is pre-scaled by 2^-16 so that w * 2^111 stays finite for |q_c s_c| < 2^32 (any binary16 data);
//     the final score is scaled back by 2^16.  All scalings are powers of two: no rounding is added;
//   * base[G] = sum_c q_c * z[G][c] is reduced inside each row with DPP rotates.
//
// Channel bookkeeping.  Meta: lane n of a row loads (s,z) of channels 4n..4n+3 and 64+4n..64+4n+3 as two
// 16-byte requests: register m = 4h + e holds channel c = 64h + 4n + e.  Bits: channel c sits in word
// d = h + 2(e & 1) at bit i = 2n + (e >> 1).  Bit i is tested in rotation a = ((i - 27) mod 32) / 4 at
// position 27 + ((i - 27) mod 4).
#include "fier_dev.h"
#include "fier_kernels.h"
#include "fier_quant_dev.h"

// MFMA variant of the inner product (the default).  The contraction over the 128 channels runs on the matrix
// cores with the 1-bit codes as the B operand and the per-group weights as the A operand of
// v_mfma_f32_16x16x32_bf16:
//   * B (bits): a bfloat16 whose only set bit is exponent bit e IS the number 2^(2^e - 127); one v_and of the code
//     word with a two-bit mask therefore yields two B elements (one per 16-bit half), eight masks cover bits
//     7..14 / 23..30 of a word and one rotation by 8 the other sixteen bits: 17 vector ops per 32 elements instead
//     of 2.2 per element.  Lane (n, kq) of the wavefront owns word kq of token n of a 16-token tile;
//   * A (weights): w = q_c s_c times the inverse of its bit's power of two (and 2^-32 against overflow), split
//     exactly into three bfloat16 terms (8 + 8 + 8 significand bits), one matrix row per term: rows 0-2 carry the
//     first group of the pair block, rows 8-10 the second.  The rows are built once per pair block by the lanes
//     that hold the group's (s, z) and handed to the A layout through 4 KiB of LDS per wavefront;
//   * every product is exact (one factor is a power of two), the matrix core accumulates in binary32, and the
//     three rows of a group are added at the end: the result is the same fp32 sum, in another order.
namespace fier {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr bool kScoreUseMfma = true;

constexpr int kScorePairsPerWave = kRangeTokens / 256;  // pair blocks per wavefront (4 wavefronts per workgroup)

__device__ __forceinline__ uint32_t rotr32(uint32_t x, int r) { return __builtin_amdgcn_alignbit(x, x, r); }

// 2^-16 / (value of a binary32 whose only set bit is bit 27 + j)
__device__ __forceinline__ float position_scale(int j) {
  // j = 0: 2^111, 1: 2^95, 2: 2^63, 3: 2^-1, each times 2^-16
  const uint32_t e = j == 0 ? (127u + 95u) : j == 1 ? (127u + 79u) : j == 2 ? (127u + 47u) : (127u - 17u);
  return __uint_as_float(e << 23);
}

// Four channels (h, n, e = 0..3):  acc_e += bit ? X[4h+e] broadcast from row lane n : 0
template <int H, int N>
__device__ __forceinline__ void accumulate_4(const uint32_t (&V)[4][8], const float (&X)[8], float (&acc)[4]) {
  constexpr int I0 = 2 * N, I1 = 2 * N + 1;
  constexpr int R0 = (I0 + 32 - 27) % 32, R1 = (I1 + 32 - 27) % 32;
  constexpr int A0 = R0 / 4, A1 = R1 / 4;
  constexpr uint32_t M0 = 1u << (27 + R0 % 4), M1 = 1u << (27 + R1 % 4);
  uint32_t t0, t1;
  asm("v_and_b32 %[t0], %[m0], %[va]\n\t"
      "v_and_b32 %[t1], %[m0], %[vb]\n\t"
      "v_fmac_f32_dpp %[a0], %[x0], %[t0] row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_and_b32 %[t0], %[m1], %[vc]\n\t"
      "v_fmac_f32_dpp %[a1], %[x1], %[t1] row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_and_b32 %[t1], %[m1], %[vd]\n\t"
      "v_fmac_f32_dpp %[a2], %[x2], %[t0] row_newbcast:%[bc] row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %[a3], %[x3], %[t1] row_newbcast:%[bc] row_mask:0xf bank_mask:0xf"
      : [t0] "=&v"(t0), [t1] "=&v"(t1), [a0] "+&v"(acc[0]), [a1] "+&v"(acc[1]), [a2] "+&v"(acc[2]),
        [a3] "+&v"(acc[3])
      : [va] "v"(V[H][A0]), [vb] "v"(V[H + 2][A0]), [vc] "v"(V[H][A1]), [vd] "v"(V[H + 2][A1]), [x0] "v"(X[4 * H]),
        [x1] "v"(X[4 * H + 1]), [x2] "v"(X[4 * H + 2]), [x3] "v"(X[4 * H + 3]), [m0] "s"(M0), [m1] "s"(M1),
        [bc] "n"(N));
}

template <int H, int N>
__device__ __forceinline__ void accumulate_from(const uint32_t (&V)[4][8], const float (&X)[8], float (&acc)[4]) {
  if constexpr (H < 2) {
    accumulate_4<H, N>(V, X, acc);
    if constexpr (N + 1 < 16)
      accumulate_from<H, N + 1>(V, X, acc);
    else
      accumulate_from<H + 1, 0>(V, X, acc);
  }
}

__device__ __forceinline__ float wave_allsum(float x) {
  x = row_allsum(x);
  x += __shfl_xor(x, 16, 64);
  x += __shfl_xor(x, 32, 64);
  return x;
}

// grid (ceil(max_ctx / 1024) [+ 1 if HIST], units), block 256: workgroup x owns tokens [1024 x, 1024 x + 1024) of
// its unit, wave w the pair blocks 16 x + w, + 4, + 8, + 12.
//
// HIST (first kernel of the fused step): every score is also counted in an equal-width histogram of kSelBins
// bins over [-R, R], R = sum_c |q_c| * absmax_c >= |score| -- a bound known before any score exists, so that
// scoring and histogramming are one pass.  The workgroup's LDS histogram is added to the unit's histogram in
// memory; the unit's last workgroup reads the total, finds the bin that holds the budget-th largest score,
// publishes it and clears the histogram for the next call.
// The extra workgroup of a unit performs the decode-stage append (Sec. 3.1) when k_new is given: one wavefront
// writes the new K/V rows, re-quantizes the group the row falls in and scores that group's tokens straight from
// its registers; the other workgroups leave those tokens alone.  The bound R uses the absmax of before the
// append (every workgroup must bin with the same R); the new group's contribution is handed to the last kernel
// of the step through `newmax`.  A score outside [-R, R] simply lands in the outermost bin.
template <int DT, int NREP, bool HIST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(HIST ? 5 : 4))) void score_kernel(const uint4* kbits, const uint4* kmeta,
                                                    const float* __restrict__ kabsmax, const uint16_t* __restrict__ q,
                                                    const int32_t* __restrict__ seq_lens, int extra,
                                                    float* __restrict__ scores, UnitCtl* __restrict__ ctl,
                                                    uint32_t* __restrict__ ghist, const int32_t* __restrict__ budgets,
                                                    int max_budget, uint32_t* K, uint32_t* V,
                                                    const uint32_t* __restrict__ k_new,
                                                    const uint32_t* __restrict__ v_new, float* __restrict__ newmax,
                                                    int n_kv_heads, int max_ctx) {
  __shared__ uint32_t lhist[HIST ? kSelBins : 1];
  __shared__ __attribute__((aligned(16))) uint16_t a_lds[kScoreUseMfma ? 4 * 4 * 16 * 32 : 8];  // [wave][j][row][k]
  __shared__ uint32_t scan_tmp[4];
  __shared__ uint32_t flag;
  __shared__ int found[2];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int unit = blockIdx.y;
  const int b = unit / n_kv_heads;
  int Lold = seq_lens[b];
  Lold = Lold < 0 ? 0 : (Lold > max_ctx ? max_ctx : Lold);
  const bool app = HIST && k_new != nullptr && Lold < max_ctx;  // this unit receives a new row in this step
  int L = HIST ? Lold + (app ? 1 : 0) : Lold + extra;
  L = L > max_ctx ? max_ctx : L;
  const int tail_start = app ? (Lold / kG) * kG : L;  // tokens from here on are scored by the appending wave
  // HIST: workgroup 0 is the appending one (dispatched first: its single wavefront has the longest chain of
  // dependent loads), workgroups 1.. score the ranges 0..
  const bool append_wg = HIST && blockIdx.x == 0;
  const int range = (int)blockIdx.x - (HIST ? 1 : 0);
  if (append_wg) {
    if (!app) return;
  } else {
    // range 0 of a unit always runs so that an empty unit still gets its control block written
    if (range * kRangeTokens >= L && !(HIST && range == 0)) return;
  }
  const int n_groups = max_ctx / kG;
  const int row = lane >> 4, n = lane & 15;
  FIER_PROF(0, HIST && unit == 0 && range == 3)
  FIER_PROF(7, HIST && unit == 0 && append_wg)
  FIER_PROF(26, HIST && unit == (int)gridDim.y - 1 && range == 30)
  FIER_PROF(28, HIST && unit == (int)gridDim.y / 2 && range == 16)

  // The lane's 8 query channels, summed over the query heads that share this kv head (binary32), times
  // 2^-16: qz for the offsets, qx additionally times the inverse of the power of two its bit is tested at.
  float qx[8], qz[8];
  float R = 0.f, hscale = 0.f;
  const uint16_t* qb = q + (size_t)unit * NREP * kD;
  {
    float rpart = 0.f;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int e = m & 3;
      const int c = 64 * (m >> 2) + 4 * n + e;
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < NREP; ++r) s += w2f<DT>(qb[r * kD + c]);
      const int i = 2 * n + (e >> 1);
      qz[m] = s * 1.52587890625e-05f;
      qx[m] = s * position_scale((i + 32 - 27) & 3);
      if (HIST) rpart += fabsf(s) * kabsmax[(size_t)unit * kD + c];
    }
    if (HIST) {
      // every row holds all 128 channels; lane 0's sum is taken so that R is bit-identical in every lane, wave
      // and workgroup (the binning must be the same function everywhere)
      R = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(row_allsum(rpart))));
      hscale = (float)kSelBins / (R + R);
      for (int i = tid; i < kSelBins; i += 256) lhist[i] = 0;
      __syncthreads();
    }
  }

  FIER_PROF(1, HIST && unit == 0 && range == 3)
  if (append_wg) {
    if constexpr (HIST) {
      if (wave == 0) {  // lane = channel pair (2 lane, 2 lane + 1)
        const uint32_t kn = k_new[(size_t)unit * (kD / 2) + lane];
        const uint32_t vn = v_new[(size_t)unit * (kD / 2) + lane];
        GroupCode gc;
        int t0, ntok;
        append_row<DT>(K, V, const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kbits)),
                       const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(kmeta)), unit, Lold, max_ctx, kn, vn,
                       lane, gc, t0, ntok);
        newmax[(size_t)unit * kD + 2 * lane] = gc.amax_lo;
        newmax[(size_t)unit * kD + 2 * lane + 1] = gc.amax_hi;
        float q0 = 0.f, q1 = 0.f;
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
          q0 += w2f<DT>(qb[r * kD + 2 * lane]);
          q1 += w2f<DT>(qb[r * kD + 2 * lane + 1]);
        }
        const float w0 = q0 * gc.s_lo, w1 = q1 * gc.s_hi;
        const float base = wave_allsum(q0 * gc.z_lo + q1 * gc.z_hi);
        float mine = 0.f;
#pragma unroll
        for (int t = 0; t < kG; ++t) {
          float v = ((gc.bits_lo >> t) & 1u ? w0 : 0.f) + ((gc.bits_hi >> t) & 1u ? w1 : 0.f);
          v = wave_allsum(v);
          if (lane == t) mine = v + base;
        }
        if (lane < ntok) {
          scores[(size_t)unit * max_ctx + t0 + lane] = mine;
          atomicAdd(&lhist[sel_bin(mine, R, hscale, kSelBins)], 1u);
        }
      }
    }
  }

  const int P0 = range * (4 * kScorePairsPerWave) + wave;  // this wave's blocks: P0, P0 + 4, ...
  if constexpr (kScoreUseMfma) {
    // zero this wave's A buffer once: the rows that carry no weights must read as zero
    {
      uint4* az = reinterpret_cast<uint4*>(a_lds) + wave * 256;
#pragma unroll
      for (int k = 0; k < 4; ++k) az[lane + 64 * k] = make_uint4(0, 0, 0, 0);
    }
    if (!append_wg && P0 * kPair < L) {
      const uint32_t* __restrict__ bits_u = reinterpret_cast<const uint32_t*>(kbits) + (size_t)unit * max_ctx * 4;
      const uint4* __restrict__ meta_u = kmeta + (size_t)unit * n_groups * (kD / 4);
      const int gsel = row >> 1;   // the group whose (s, z) this row of lanes holds
      const int hsel = row & 1;    // the 64-channel half whose weights this row converts
      // per-lane constants of the weight rows: channel c_e = 64 hsel + 4n + e sits in word kq_c at bit i_c
      float qf[4];
      int a_off[4];  // byte offset of the first (most significant) term of channel e in this wave's A buffer
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int kq_c = hsel + 2 * (e & 1);
        const int i_c = 2 * n + (e >> 1);
        int v, hf, p;
        if (i_c >= 7 && i_c <= 14) {
          v = 0, hf = 0, p = i_c;
        } else if (i_c >= 23 && i_c <= 30) {
          v = 0, hf = 1, p = i_c - 16;
        } else if (i_c >= 15 && i_c <= 22) {
          v = 1, hf = 0, p = i_c - 8;
        } else {
          v = 1, hf = 1, p = (i_c + 8) & 31;
        }
        const int j = 2 * v + ((p - 7) >> 2), r = (p - 7) & 3, k = 8 * kq_c + 2 * r + hf;
        // 2^-32 / (value of a bfloat16 whose only set bit is bit p) = 2^(95 - 2^(p-7))
        const float comp = __uint_as_float((uint32_t)(127 + 95 - (1 << (p - 7))) << 23);
        qf[e] = qz[4 * hsel + e] * 65536.0f * comp;  // qz holds q * 2^-16
        a_off[e] = wave * 4096 + j * 1024 + (8 * gsel) * 64 + k * 2;
      }
      float qb8[8];  // q * 2^-32 for the offsets z
#pragma unroll
      for (int m = 0; m < 8; ++m) qb8[m] = qz[m] * 1.52587890625e-05f;

      uint32_t w_cur[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) w_cur[t] = bits_u[(size_t)(P0 * kPair + 16 * t + n) * 4 + row];
      uint4 ma_cur = meta_u[(size_t)(2 * P0 + gsel) * (kD / 4) + n];
      uint4 mb_cur = meta_u[(size_t)(2 * P0 + gsel) * (kD / 4) + 16 + n];
      char* a_bytes = reinterpret_cast<char*>(a_lds);

#pragma unroll 1
      for (int it = 0; it < kScorePairsPerWave; ++it) {
        const int P = P0 + 4 * it;
        if (P * kPair >= L) break;
        int Pn = P + 4;
        Pn = (it + 1 < kScorePairsPerWave && Pn * kPair < L) ? Pn : P;
        uint32_t w_nxt[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) w_nxt[t] = bits_u[(size_t)(Pn * kPair + 16 * t + n) * 4 + row];
        const uint4 ma_nxt = meta_u[(size_t)(2 * Pn + gsel) * (kD / 4) + n];
        const uint4 mb_nxt = meta_u[(size_t)(2 * Pn + gsel) * (kD / 4) + 16 + n];

        // ---- weight rows of this row's group and channel half -> LDS ----------------------------------------
        const uint32_t mwa[4] = {ma_cur.x, ma_cur.y, ma_cur.z, ma_cur.w};
        const uint32_t mwb[4] = {mb_cur.x, mb_cur.y, mb_cur.z, mb_cur.w};
        float basep = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          basep += qb8[e] * hi16f<DT>(mwa[e]);
          basep += qb8[4 + e] * hi16f<DT>(mwb[e]);
          const float sv = lo16f<DT>(hsel ? mwb[e] : mwa[e]);
          const float w = qf[e] * sv;
          const uint32_t wb = __float_as_uint(w);
          const float r1 = w - __uint_as_float(wb & 0xffff0000u);
          const uint32_t r1b = __float_as_uint(r1);
          const float r2 = r1 - __uint_as_float(r1b & 0xffff0000u);
          *reinterpret_cast<uint16_t*>(a_bytes + a_off[e]) = (uint16_t)(wb >> 16);
          *reinterpret_cast<uint16_t*>(a_bytes + a_off[e] + 64) = (uint16_t)(r1b >> 16);
          *reinterpret_cast<uint16_t*>(a_bytes + a_off[e] + 128) = (uint16_t)(__float_as_uint(r2) >> 16);
        }
        const float base = row_allsum(basep);  // every row holds all 128 offsets of its group
        // the writes above come from other lanes of this same wavefront: LDS operations of a wavefront complete
        // in order, the fence keeps the compiler from moving the reads above them
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        bf16x8_t areg[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          areg[j] = __builtin_bit_cast(
              bf16x8_t, *reinterpret_cast<const u32x4_t*>(a_bytes + wave * 4096 + j * 1024 + n * 64 + row * 16));
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // reads done before the next block's writes

        // ---- four 16-token tiles: bits -> B operand, 4 MFMAs each -------------------------------------------
        floatx4_t acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint32_t word = (j >> 1) ? rotr32(w_cur[t], 8) : w_cur[t];
            u32x4_t b;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int p = 7 + 4 * (j & 1) + r;
              b[r] = word & ((1u << p) | (1u << (p + 16)));
            }
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[j], __builtin_bit_cast(bf16x8_t, b), acc[t], 0, 0, 0);
          }
        }
        // rows 0-2 (lanes 0-15) hold the first group's tiles 0, 1; rows 8-10 (lanes 32-47) the second group's 2, 3
        const bool second = row == 2;
        const floatx4_t da = second ? acc[2] : acc[0], db = second ? acc[3] : acc[1];
        const float sa = (((da[0] + da[1]) + da[2]) + base) * 4294967296.0f;
        const float sb = (((db[0] + db[1]) + db[2]) + base) * 4294967296.0f;
        if ((row & 1) == 0) {
          const int tok = P * kPair + 16 * row + n;  // row 0: tokens n, 16 + n; row 2: 32 + n, 48 + n
          if (tok < L && tok < tail_start) {
            scores[(size_t)unit * max_ctx + tok] = sa;
            if (HIST) atomicAdd(&lhist[sel_bin(sa, R, hscale, kSelBins)], 1u);
          }
          if (tok + 16 < L && tok + 16 < tail_start) {
            scores[(size_t)unit * max_ctx + tok + 16] = sb;
            if (HIST) atomicAdd(&lhist[sel_bin(sb, R, hscale, kSelBins)], 1u);
          }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) w_cur[t] = w_nxt[t];
        ma_cur = ma_nxt;
        mb_cur = mb_nxt;
      }
    }
  } else {
  if (!append_wg && P0 * kPair < L) {
    const uint4* __restrict__ bits_u = kbits + (size_t)unit * max_ctx;
    const uint4* __restrict__ meta_u = kmeta + (size_t)unit * n_groups * (kD / 4);
    const int gsel = row >> 1;

    uint4 w_cur = bits_u[P0 * kPair + lane];
    uint4 ma_cur = meta_u[(size_t)(2 * P0 + gsel) * (kD / 4) + n];
    uint4 mb_cur = meta_u[(size_t)(2 * P0 + gsel) * (kD / 4) + 16 + n];

#pragma unroll 1
    for (int it = 0; it < kScorePairsPerWave; ++it) {
      const int P = P0 + 4 * it;
      if (P * kPair >= L) break;
      // prefetch the next block of this wave (clamped to stay inside the unit's buffers)
      int Pn = P + 4;
      Pn = (it + 1 < kScorePairsPerWave && Pn * kPair < L) ? Pn : P;
      const uint4 w_nxt = bits_u[Pn * kPair + lane];
      const uint4 ma_nxt = meta_u[(size_t)(2 * Pn + gsel) * (kD / 4) + n];
      const uint4 mb_nxt = meta_u[(size_t)(2 * Pn + gsel) * (kD / 4) + 16 + n];

      const uint32_t mw[8] = {ma_cur.x, ma_cur.y, ma_cur.z, ma_cur.w, mb_cur.x, mb_cur.y, mb_cur.z, mb_cur.w};
      float X[8];
      float basep = 0.f;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        X[m] = qx[m] * lo16f<DT>(mw[m]);
        basep += qz[m] * hi16f<DT>(mw[m]);
      }
      const uint32_t ww[4] = {w_cur.x, w_cur.y, w_cur.z, w_cur.w};
      uint32_t V[4][8];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        V[d][0] = ww[d];
#pragma unroll
        for (int a = 1; a < 8; ++a) V[d][a] = rotr32(ww[d], 4 * a);
      }
      const float base = row_allsum(basep);
      // A DPP source must not be read within two issue slots of the VALU write that produced it.  The weights
      // pass through this fence so that every later DPP read of them is at least that far from their writes.
      asm volatile("s_nop 1"
                   : "+v"(X[0]), "+v"(X[1]), "+v"(X[2]), "+v"(X[3]), "+v"(X[4]), "+v"(X[5]), "+v"(X[6]), "+v"(X[7]));
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      accumulate_from<0, 0>(V, X, acc);
      const float sc = (((acc[0] + acc[1]) + (acc[2] + acc[3])) + base) * 65536.0f;
      const int tok = P * kPair + lane;
      if (tok < L && tok < tail_start) {
        scores[(size_t)unit * max_ctx + tok] = sc;
        if (HIST) atomicAdd(&lhist[sel_bin(sc, R, hscale, kSelBins)], 1u);
      }
      w_cur = w_nxt;
      ma_cur = ma_nxt;
      mb_cur = mb_nxt;
    }
  }

  }

  FIER_PROF(2, HIST && unit == 0 && range == 3)
  FIER_PROF(8, HIST && unit == 0 && append_wg)
  FIER_PROF(27, HIST && unit == (int)gridDim.y - 1 && range == 30)
  FIER_PROF(29, HIST && unit == (int)gridDim.y / 2 && range == 16)
  if constexpr (HIST) {
    __syncthreads();
    uint32_t* __restrict__ gh = ghist + (size_t)unit * kSelBins;
    for (int i = tid; i < kSelBins; i += 256) {
      const uint32_t c = lhist[i];
      if (c) atomicAdd(&gh[i], c);
    }
    const uint32_t expected = (L > 0 ? (uint32_t)((L + kRangeTokens - 1) / kRangeTokens) : 1u) + (app ? 1u : 0u);
    FIER_PROF(3, unit == 0 && range == 3)
    if (!last_arriver(&ctl[unit].arrive[0], expected, &flag)) return;
    FIER_PROF(4, unit == 0)
    // ---- the unit's last workgroup: threshold bin for the budget ---------------------------------------
    int B = budgets[b];
    B = B > max_budget ? max_budget : B;
    B = B > L ? L : B;
    B = B < 0 ? 0 : B;
    constexpr int PER = kSelBins / 256;
    // thread t owns bins kSelBins-1-PER*t down to kSelBins-PER*(t+1), i.e. descending score order
    uint32_t cnt[PER], sum = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      cnt[k] = load_coherent(&gh[kSelBins - 1 - (PER * tid + k)]);
      sum += cnt[k];
    }
    uint32_t total;
    uint32_t before = block_excl_scan_u32<4>(sum, scan_tmp, total);
    if (tid == 0) {
      found[0] = B >= L ? -1 : kSelBins;  // everything / nothing selected by bin alone
      found[1] = 0;
    }
    __syncthreads();
    if (B > 0 && B < L) {
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        if (before < (uint32_t)B && (uint32_t)B <= before + cnt[k]) {
          found[0] = kSelBins - 1 - (PER * tid + k);
          found[1] = (int)before;
        }
        before += cnt[k];
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < PER; ++k) gh[kSelBins - 1 - (PER * tid + k)] = 0;
    if (tid == 0) {
      UnitCtl* c = &ctl[unit];
      c->tbin = found[0];
      c->above = (uint32_t)found[1];
      c->budget = B;
      c->R = R;
      c->scale = hscale;
      c->arrive[0] = 0;
    }
    FIER_PROF(5, unit == 0)
  }
}

template <int DT, bool HIST>
static hipError_t launch_score_dt(int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                                  const void* q, const int32_t* seq_lens, int extra, float* scores,
                                  const StepBuffers* sb, const int32_t* budgets, int max_budget, void* K, void* V,
                                  const void* k_new, const void* v_new, int units, int n_kv_heads, int max_ctx,
                                  hipStream_t st) {
  dim3 grid((max_ctx + kRangeTokens - 1) / kRangeTokens + (HIST ? 1 : 0), units);
#define FIER_SCORE_CASE(R)                                                                                         \
  case R:                                                                                                          \
    score_kernel<DT, R, HIST><<<grid, 256, 0, st>>>(                                                               \
        (const uint4*)kbits, (const uint4*)kmeta, kabsmax, (const uint16_t*)q, seq_lens, extra, scores,            \
        sb ? sb->ctl : nullptr, sb ? sb->hist : nullptr, budgets, max_budget, (uint32_t*)K, (uint32_t*)V,          \
        (const uint32_t*)k_new, (const uint32_t*)v_new, sb ? sb->newmax : nullptr, n_kv_heads, max_ctx);           \
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

hipError_t launch_score(int dtype, int n_rep, const uint32_t* kbits, const uint32_t* kmeta, const float* kabsmax,
                        const void* q, const int32_t* seq_lens, int extra, float* scores, const StepBuffers* sb,
                        const int32_t* budgets, int max_budget, void* K, void* V, const void* k_new,
                        const void* v_new, int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  if (sb) {
    if (dtype == DT_F16)
      return launch_score_dt<DT_F16, true>(n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, sb, budgets,
                                           max_budget, K, V, k_new, v_new, units, n_kv_heads, max_ctx, st);
    return launch_score_dt<DT_BF16, true>(n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, sb, budgets,
                                          max_budget, K, V, k_new, v_new, units, n_kv_heads, max_ctx, st);
  }
  if (dtype == DT_F16)
    return launch_score_dt<DT_F16, false>(n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, nullptr, nullptr,
                                          0, nullptr, nullptr, nullptr, nullptr, units, n_kv_heads, max_ctx, st);
  return launch_score_dt<DT_BF16, false>(n_rep, kbits, kmeta, kabsmax, q, seq_lens, extra, scores, nullptr, nullptr, 0,
                                         nullptr, nullptr, nullptr, nullptr, units, n_kv_heads, max_ctx, st);
}

}  // namespace fier
