// The 1-bit group quantizer as a device function, shared by the bulk quantizer, the append kernel and the
// fused decode step (Alg. 1 step 1; Eq. 5 read as round-to-nearest, Sec. 3.3).
#pragma once

#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

struct GroupCode {          // what one lane (channels 2l, 2l+1) learns about a group
  uint32_t meta_lo, meta_hi;  // s | z << 16 in the K dtype
  float s_lo, z_lo, s_hi, z_hi;  // the same as binary32
  float amax_lo, amax_hi;     // max(|z|, |z + s|): the larger reconstruction level in magnitude
  uint32_t bits_lo, bits_hi;  // bit t = code of token t (channel-major view of the group)
};

// ---- the decision arithmetic, in one place (binary32, no contraction) --------------------------------------------
// z = min (-0 -> +0);  s = RN_dtype(max - z), held at the largest finite value;  bit = 2 * (k - z) >= s.
struct MinMax {  // running min / max of the lane's two channels over the tokens seen so far
  float mn0, mx0, mn1, mx1;
};
template <int DT>
__device__ __forceinline__ void minmax_first(MinMax& m, uint32_t row) {
  m.mn0 = m.mx0 = lo16f<DT>(row);
  m.mn1 = m.mx1 = hi16f<DT>(row);
}
template <int DT>
__device__ __forceinline__ void minmax_update(MinMax& m, uint32_t row, bool present) {
  const float a = lo16f<DT>(row), b = hi16f<DT>(row);
  m.mn0 = (present && a < m.mn0) ? a : m.mn0;
  m.mx0 = (present && a > m.mx0) ? a : m.mx0;
  m.mn1 = (present && b < m.mn1) ? b : m.mn1;
  m.mx1 = (present && b > m.mx1) ? b : m.mx1;
}
struct GroupScale {  // (s, z) of the lane's two channels: stored words and the same as binary32
  uint32_t s0, z0, s1, z1;
  float sf0, zf0, sf1, zf1;
};
template <int DT>
__device__ __forceinline__ GroupScale group_scale(MinMax m) {
#pragma clang fp contract(off)
  const float cap = DT == DT_F16 ? 65504.0f : 3.3895313892515355e38f;
  if (m.mn0 == 0.0f) m.mn0 = 0.0f;
  if (m.mn1 == 0.0f) m.mn1 = 0.0f;
  float d0 = m.mx0 - m.mn0;
  float d1 = m.mx1 - m.mn1;
  d0 = d0 > cap ? cap : d0;
  d1 = d1 > cap ? cap : d1;
  if (d0 == 0.0f) d0 = 0.0f;
  if (d1 == 0.0f) d1 = 0.0f;
  GroupScale g;
  g.s0 = f2w<DT>(d0), g.s1 = f2w<DT>(d1);
  g.z0 = f2w<DT>(m.mn0), g.z1 = f2w<DT>(m.mn1);
  g.sf0 = w2f<DT>(g.s0), g.sf1 = w2f<DT>(g.s1);
  g.zf0 = w2f<DT>(g.z0), g.zf1 = w2f<DT>(g.z1);
  return g;
}
// Codes of up to 32 rows (tokens 0..ntok-1 present; FULL: all 32, ntok is not looked at) under scale g.  Lane
// lane_base + t receives the 128-bit code word of token t in `mine`; b0 / b1 collect the lane's own two channels
// (bit t = token t).
template <int DT, bool FULL = false>
__device__ __forceinline__ void code_rows(const uint32_t (&rows)[kG], int ntok, const GroupScale& g, int lane,
                                          int lane_base, uint4& mine, uint32_t& b0, uint32_t& b1) {
#pragma clang fp contract(off)
  b0 = 0, b1 = 0;
  uint32_t r = rows[0];
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    // ntok is the same in every lane: a row that is not there costs one scalar branch, not a row's worth of work
    // (the appending wavefront of a decode step is a single wavefront on the step's critical path, and a group that
    // has just been opened holds one token)
    if (FULL || t < ntok) {
      const float a = lo16f<DT>(r) - g.zf0;
      const float b = hi16f<DT>(r) - g.zf1;
      const bool c0 = a + a >= g.sf0, c1 = b + b >= g.sf1;
      const uint64_t even = __ballot(c0);
      const uint64_t odd = __ballot(c1);
      b0 |= c0 ? (1u << t) : 0u;
      b1 |= c1 ? (1u << t) : 0u;
      if (lane == lane_base + t)
        mine = make_uint4((uint32_t)even, (uint32_t)(even >> 32), (uint32_t)odd, (uint32_t)(odd >> 32));
    }
    if (t + 1 < kG) {
      // An empty statement that "produces" the next row and `mine`: the next row's compares cannot start before
      // this row's ballots have been used up.  Left to itself the compiler makes the ballots of all 32 rows first,
      // and 64 of them do not fit the scalar registers (they were spilled to vector lanes and read back).
      r = rows[t + 1];
      asm volatile("" : "+v"(r), "+v"(mine.x), "+v"(mine.y), "+v"(mine.z), "+v"(mine.w));
    }
  }
}
template <int DT>
__device__ __forceinline__ void fill_code(GroupCode& gc, const GroupScale& g, uint32_t b0, uint32_t b1) {
  gc.meta_lo = g.s0 | (g.z0 << 16);
  gc.meta_hi = g.s1 | (g.z1 << 16);
  gc.s_lo = g.sf0;
  gc.z_lo = g.zf0;
  gc.s_hi = g.sf1;
  gc.z_hi = g.zf1;
  gc.amax_lo = fmaxf(fabsf(g.zf0), fabsf(g.zf0 + g.sf0));
  gc.amax_hi = fmaxf(fabsf(g.zf1), fabsf(g.zf1 + g.sf1));
  gc.bits_lo = b0;
  gc.bits_hi = b1;
}

// Quantize one 32-token group (ntok in [1, 32] tokens present) for the lane's two channels.
// rows[t] holds the packed pair (channel 2l in the low half) of token t; entries t >= ntok are ignored.
// Lane lane_base + t receives the 128-bit code word of token t in `mine` (zero for tokens not present):
// x, y = even channels 0..62 / 64..126 (bit i = channel 2i, 64 + 2i), z, w = odd channels likewise.
template <int DT>
__device__ __forceinline__ void quantize_group(const uint32_t (&rows)[kG], int ntok, int lane, int lane_base,
                                               uint4& mine, GroupCode& gc) {
  MinMax m;
  minmax_first<DT>(m, rows[0]);
#pragma unroll
  for (int t = 1; t < kG; ++t)
    if (t < ntok) minmax_update<DT>(m, rows[t], true);  // the same in every lane: a scalar branch per absent row
  const GroupScale g = group_scale<DT>(m);
  uint32_t b0, b1;
  code_rows<DT>(rows, ntok, g, lane, lane_base, mine, b0, b1);
  fill_code<DT>(gc, g, b0, b1);
}

// Groups of g = 32 ns tokens, ns in {2, 4, 8}: the group's rows do not fit the registers, so they are read twice
// (min / max, then codes), 32 rows at a time.  row_at(t) returns the packed pair of token t of the group (t < ntok).
// Pass 1 returns the scale; pass 2 is code_rows per 32-token chunk, driven by the caller.
template <int DT, class RowAt>
__device__ __forceinline__ GroupScale long_group_scale(RowAt row_at, int ntok) {
  MinMax m;
  minmax_first<DT>(m, row_at(0));
  for (int c0 = 0; c0 < ntok; c0 += kG) {
    uint32_t rows[kG];
#pragma unroll
    for (int t = 0; t < kG; ++t) rows[t] = row_at(c0 + t < ntok ? c0 + t : 0);
#pragma unroll
    for (int t = 0; t < kG; ++t) minmax_update<DT>(m, rows[t], c0 + t < ntok);
  }
  return group_scale<DT>(m);
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
__device__ __forceinline__ void append_load_rows(const uint32_t* __restrict__ K, const KvRows kv, int L, uint32_t kn,
                                                 int lane, uint32_t (&rows)[kG], int& t0, int& ntok) {
  const int Gi = L / kG;
  t0 = Gi * kG;
  ntok = L - t0 + 1;
  const uint32_t* src = K + kv.row(t0) * (kD / 2) + lane;  // a group lies inside one block
#pragma unroll
  for (int t = 0; t < kG; ++t) {
    // rows before the new one come from memory (t0 + t < L: never the row the append writes)
    uint32_t r = t < ntok - 1 ? src[(size_t)t * (kD / 2)] : 0u;
    rows[t] = (t == ntok - 1) ? kn : r;
  }
}

// rows, t0, ntok: from append_load_rows (which may run well before: the loads are the long part of the chain)
template <int DT>
__device__ __forceinline__ void append_finish(uint32_t* __restrict__ K, uint32_t* __restrict__ V, const KvRows kv,
                                              uint32_t* __restrict__ kbits, uint32_t* __restrict__ kmeta, int unit,
                                              int L, int max_ctx, uint32_t kn, uint32_t vn, int lane,
                                              const uint32_t (&rows)[kG], int t0, int ntok, GroupCode& gc,
                                              uint4& mine) {
  const int n_groups = max_ctx / kG;
  K[kv.row(L) * (kD / 2) + lane] = kn;
  V[kv.row(L) * (kD / 2) + lane] = vn;
  const int Gi = L / kG;
  mine = make_uint4(0, 0, 0, 0);
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

template <int DT>
__device__ __forceinline__ void append_row(uint32_t* __restrict__ K, uint32_t* __restrict__ V, const KvRows kv,
                                           uint32_t* __restrict__ kbits, uint32_t* __restrict__ kmeta, int unit,
                                           int L, int max_ctx, uint32_t kn, uint32_t vn, int lane, GroupCode& gc,
                                           int& t0, int& ntok, uint4& mine) {
  uint32_t rows[kG];
  append_load_rows<DT>(K, kv, L, kn, lane, rows, t0, ntok);
  append_finish<DT>(K, V, kv, kbits, kmeta, unit, L, max_ctx, kn, vn, lane, rows, t0, ntok, gc, mine);
}

// The same for groups of g = 32 ns tokens (ns in {2, 4, 8}): the tail group (up to g rows) is read twice, 32 rows at a
// time.  Every pair block of the group that holds a token gets its code words rewritten; on_block(pb, mine, gs)
// is called once per such block with the calling lane's code word of token t0 + 64 pb + lane (zero if absent) and the
// group's scale.
template <int DT, class OnBlock>
__device__ __forceinline__ GroupScale append_row_long(uint32_t* __restrict__ K, uint32_t* __restrict__ V,
                                                      const KvRows kv, uint32_t* __restrict__ kbits,
                                                      uint32_t* __restrict__ kmeta,
                                                      int unit, int L, int max_ctx, int ns, uint32_t kn, uint32_t vn,
                                                      int lane, int& t0, int& ntok, OnBlock on_block) {
  const int g = kG * ns;
  const int n_groups = max_ctx / g;
  K[kv.row(L) * (kD / 2) + lane] = kn;
  V[kv.row(L) * (kD / 2) + lane] = vn;
  const int Gi = L / g;
  t0 = Gi * g;
  ntok = L - t0 + 1;
  const int n_present = ntok;
  const uint32_t* src = K + kv.row(t0) * (kD / 2) + lane;  // a group lies inside one block
  // rows before the new one come from memory (never the row written above), the new one from registers
  auto row_at = [&](int t) { return t == n_present - 1 ? kn : src[(size_t)t * (kD / 2)]; };
  const GroupScale gs = long_group_scale<DT>(row_at, ntok);
  uint2* mdst = reinterpret_cast<uint2*>(kmeta + ((size_t)unit * n_groups + Gi) * kD) + lane;
  *mdst = make_uint2(gs.s0 | (gs.z0 << 16), gs.s1 | (gs.z1 << 16));
  uint4* bdst = reinterpret_cast<uint4*>(kbits) + (size_t)unit * max_ctx + t0;
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
    bdst[pb * kPair + lane] = mine;
    on_block(pb, mine, gs);
  }
  return gs;
}

}  // namespace fier
