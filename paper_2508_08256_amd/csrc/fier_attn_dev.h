// Device functions of the attention kernels (Alg. 1 step 4): the gather loops over a row list, the per-workgroup
// partial (m, l, o) store and the merge of a unit's partials.  Shared by the stand-alone attention kernel
// (fier_attn.hip) and the fused decode step (fier_step.hip).
#pragma once

#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

constexpr int kAttnUnroll = 2;                  // rows per 16-lane row per iteration
constexpr int kRowsPerIter = 4 * 4 * kAttnUnroll;  // 4 waves x 4 lane rows x unroll

// Running softmax state of one 16-lane row of a wavefront, per query head: lane cn holds channels 8cn..8cn+7.
template <int NREP>
struct AttnState {
  float m[NREP], l[NREP], o[NREP][8];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
      m[r] = -INFINITY;
      l[r] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[r][c] = 0.f;
    }
  }
};

// A row_of that cannot place an entry (an index outside the cache in a caller's list) returns this; the entry is
// then skipped: it gets no weight.
constexpr size_t kNoRow = ~(size_t)0;



// Attend over entries [start, end) of a row list; row_of(j) gives the row of entry j in the K / V arrays (the
// callers map a token to its row: contiguous, or through the block table), or kNoRow if CHECKED and the entry
// is to be skipped (safe_row is then read in its place and masked).  The workgroup's
// 16 lane rows (4 waves x 4) take entries round-robin in batches of kAttnUnroll.  Calls may follow each other
// on the same state: the running softmax simply continues.
template <int DT, int NREP, bool CHECKED = false, bool STREAM = false, class RowOf>
__device__ __forceinline__ void attend_rows(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                            const uint4 (&qr)[NREP], RowOf row_of, int start, int end,
                                            float scale_log2e, AttnState<NREP>& st, size_t safe_row = 0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rs = lane >> 4, cn = lane & 15;
  for (int i0 = start + wave * (4 * kAttnUnroll); i0 < end; i0 += kRowsPerIter) {
    uint4 kk[kAttnUnroll], vv[kAttnUnroll];
    bool valid[kAttnUnroll];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int j = i0 + u * 4 + rs;
      valid[u] = j < end;
      size_t r = row_of(valid[u] ? j : start);
      if (CHECKED) {
        valid[u] = valid[u] && r != kNoRow;
        r = r == kNoRow ? safe_row : r;
      }
      const size_t ro = r * (kD / 8) + cn;
      kk[u] = STREAM ? load_stream(K + ro) : K[ro];
      vv[u] = STREAM ? load_stream(V + ro) : V[ro];
    }
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
      float logit[kAttnUnroll];
      float mx = st.m[r];
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        float d = dot2<DT>(kk[u].x, qr[r].x, 0.f);
        d = dot2<DT>(kk[u].y, qr[r].y, d);
        d = dot2<DT>(kk[u].z, qr[r].z, d);
        d = dot2<DT>(kk[u].w, qr[r].w, d);
        d = row_allsum(d);
        logit[u] = valid[u] ? d * scale_log2e : -INFINITY;
        mx = fmaxf(mx, logit[u]);
      }
      const float mref = mx == -INFINITY ? 0.f : mx;
      const float alpha = __builtin_amdgcn_exp2f(st.m[r] - mref);
      float p[kAttnUnroll], psum = 0.f;
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        p[u] = __builtin_amdgcn_exp2f(logit[u] - mref);
        psum += p[u];
      }
      st.m[r] = mx;
      st.l[r] = st.l[r] * alpha + psum;
#pragma unroll
      for (int c = 0; c < 8; ++c) st.o[r][c] *= alpha;
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        const uint32_t vw[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          st.o[r][2 * c] += p[u] * lo16f<DT>(vw[c]);
          st.o[r][2 * c + 1] += p[u] * hi16f<DT>(vw[c]);
        }
      }
    }
  }
}

typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

template <int DT>
__device__ __forceinline__ floatx4_t mfma_16x16x32(const uint4& a, const uint4& b, floatx4_t c) {
  if (DT == DT_F16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0,
                                                  0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}

constexpr int kPartialFloats = 4 * 16 * 10;  // LDS floats per query head: [wave][channel chunk][o[8], m, l]
constexpr int kAttnMfmaLds = 4 * 144;  // LDS floats attend_rows_mfma needs: per wavefront p[16 tokens][8 heads], alpha[8]

// The same for 3 to 8 query heads per kv head, where q.K^T for all heads of the group is a real (if skinny) dense
// contraction: per wavefront and 16 gathered rows, S[head][token] comes from four v_mfma_f32_16x16x32 (A = the
// queries, one matrix row per head, B = the K rows as they lie in memory: lane (n, kq) loads channels
// 32c + 8kq .. + 7 of row n).  The softmax runs on S where the matrix core leaves it (lane = token, register = head),
// the probabilities go through LDS to the lanes that own the V rows (a 16-lane row owns one V row, as in
// attend_rows) and the P.V product stays on the vector ALUs.  One running (m, l) per head and wavefront.
// q_unit: the unit's NREP query rows; sh: kAttnMfmaLds floats of LDS.  resume: st holds the result of an earlier
// call by the same workgroup and the running softmax continues from it.  CHECKED / safe_row as in attend_rows.
template <int DT, int NREP, bool CHECKED = false, bool STREAM = false, bool STREAM_V = STREAM, class RowOf>
__device__ __forceinline__ void attend_rows_mfma(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                 const uint4* __restrict__ q_unit, RowOf row_of, int start, int end,
                                                 float scale_log2e, AttnState<NREP>& st, float* sh, bool resume = false,
                                                 size_t safe_row = 0) {
  static_assert(NREP >= 1 && NREP <= 8, "heads per kv head");
  static_assert(NREP * kPartialFloats >= kAttnMfmaLds || NREP < 3, "the callers lend the partials' LDS");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, kq = lane >> 4;  // matrix view: token column n, K quarter kq; result rows 4kq..4kq+3
  float* p_sh = sh + wave * 144;            // [token][8 heads], then alpha[8]
  uint4 qa[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
    qa[c] = n < NREP ? q_unit[(size_t)n * (kD / 8) + 4 * c + kq] : make_uint4(0, 0, 0, 0);
  // running max and sum of head 4kq + i in element i, the same in the 16 lanes of a lane row
  float m_run[4], l_run[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m_run[i] = -INFINITY;
    l_run[i] = 0.f;
  }
  if (resume) {
    // the state left by the earlier call: the wavefront's running maximum of head h in every lane, its running sum
    // in lane row 0; back into the matrix view (head 4kq + i in element i) through LDS
    if (lane == 0) {
#pragma unroll
      for (int h = 0; h < NREP; ++h) {
        p_sh[h] = st.m[h];
        p_sh[8 + h] = st.l[h];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4 * kq + i < NREP) {
        m_run[i] = p_sh[4 * kq + i];
        l_run[i] = p_sh[8 + 4 * kq + i];
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // reads done before the first tile's writes
  }
  for (int j0 = start + wave * 16; j0 < end; j0 += 64) {
    // K rows in the matrix view (token j0 + n), V rows in the row-owner view (tokens j0 + 4u + kq, channels 8n..8n+7)
    const int jk = j0 + n;
    bool valid = jk < end;
    uint4 kk[4], vv[4];
    size_t rk = row_of(valid ? jk : start);
    if (CHECKED) {
      valid = valid && rk != kNoRow;
      rk = rk == kNoRow ? safe_row : rk;
    }
    rk *= (kD / 8);
#pragma unroll
    for (int c = 0; c < 4; ++c) kk[c] = STREAM ? load_stream(K + rk + 4 * c + kq) : K[rk + 4 * c + kq];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int jv = j0 + 4 * u + kq;
      size_t rv = row_of(jv < end ? jv : start);
      if (CHECKED) rv = rv == kNoRow ? safe_row : rv;  // its probability is zero: the K side masks it
      vv[u] = STREAM_V ? load_stream(V + rv * (kD / 8) + n) : V[rv * (kD / 8) + n];
    }
    floatx4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c) sacc = mfma_16x16x32<DT>(qa[c], kk[c], sacc);
    float p[4], alpha[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float logit = valid ? sacc[i] * scale_log2e : -INFINITY;
      float tmax = logit;
      tmax = fmaxf(tmax, row_ror<8>(tmax));
      tmax = fmaxf(tmax, row_ror<4>(tmax));
      tmax = fmaxf(tmax, row_ror<2>(tmax));
      tmax = fmaxf(tmax, row_ror<1>(tmax));
      const float mx = fmaxf(m_run[i], tmax);
      const float mref = mx == -INFINITY ? 0.f : mx;
      alpha[i] = __builtin_amdgcn_exp2f(m_run[i] - mref);
      p[i] = __builtin_amdgcn_exp2f(logit - mref);
      l_run[i] = l_run[i] * alpha[i] + row_allsum(p[i]);
      m_run[i] = mx;
    }
    if (4 * kq < NREP) {
      *reinterpret_cast<float4*>(p_sh + n * 8 + 4 * kq) = make_float4(p[0], p[1], p[2], p[3]);
      if (n == 0) *reinterpret_cast<float4*>(p_sh + 128 + 4 * kq) = make_float4(alpha[0], alpha[1], alpha[2], alpha[3]);
    }
    // written and read by different lanes of this same wavefront: LDS operations of a wavefront complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float al[8], pw[4][8];
    {
      const float4 a0 = *reinterpret_cast<const float4*>(p_sh + 128);
      al[0] = a0.x, al[1] = a0.y, al[2] = a0.z, al[3] = a0.w;
      if (NREP > 4) {
        const float4 a1 = *reinterpret_cast<const float4*>(p_sh + 132);
        al[4] = a1.x, al[5] = a1.y, al[6] = a1.z, al[7] = a1.w;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float4 p0 = *reinterpret_cast<const float4*>(p_sh + (4 * u + kq) * 8);
        pw[u][0] = p0.x, pw[u][1] = p0.y, pw[u][2] = p0.z, pw[u][3] = p0.w;
        if (NREP > 4) {
          const float4 p1 = *reinterpret_cast<const float4*>(p_sh + (4 * u + kq) * 8 + 4);
          pw[u][4] = p1.x, pw[u][5] = p1.y, pw[u][6] = p1.z, pw[u][7] = p1.w;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // reads done before the next tile's writes
    float vf[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t vw[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        vf[u][2 * c] = lo16f<DT>(vw[c]);
        vf[u][2 * c + 1] = hi16f<DT>(vw[c]);
      }
    }
#pragma unroll
    for (int h = 0; h < NREP; ++h)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float o = st.o[h][c] * al[h];
#pragma unroll
        for (int u = 0; u < 4; ++u) o += pw[u][h] * vf[u][c];
        st.o[h][c] = o;
      }
  }
  // the per-wavefront (m, l) into the per-lane state: every lane row carries m, the first one also l
  if (4 * kq < NREP && n == 0) {
    *reinterpret_cast<float4*>(p_sh + 4 * kq) = make_float4(m_run[0], m_run[1], m_run[2], m_run[3]);
    *reinterpret_cast<float4*>(p_sh + 8 + 4 * kq) = make_float4(l_run[0], l_run[1], l_run[2], l_run[3]);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int h = 0; h < NREP; ++h) {
    st.m[h] = p_sh[h];
    st.l[h] = kq == 0 ? p_sh[8 + h] : 0.f;
  }
}

// value of the lane 16 / 32 lanes away
__device__ __forceinline__ float xor16(float x) {
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401f));
}
__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }


// Combine the 16 lane-row states of the workgroup per query head and write one partial (m, l, o[128]) per head
// into slot `slot` of the unit's partial arrays.  The four lane rows of a wavefront are folded with cross-lane
// moves first, so that only one state per wavefront and head goes through LDS and all heads share one barrier.
// sh: NREP * kPartialFloats floats.  Contains barriers: every thread of the workgroup calls it.
// mark: the slot's l goes out as -(l + 1) (l >= 0, so the sign is free): a workgroup of the step records that way that
// its partial lacks its threshold-bin rows (merge_heads takes such a slot with its true l).
template <int NREP, bool COHERENT>
__device__ __forceinline__ void store_partials(const AttnState<NREP>& st, float* sh, int unit, int n_slots, int slot,
                                               float* __restrict__ po, float* __restrict__ pm,
                                               float* __restrict__ pl, bool mark = false) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int rs = lane >> 4, cn = lane & 15;
  __syncthreads();  // sh may still be read as something else by a slower wavefront
#pragma unroll
  for (int r = 0; r < NREP; ++r) {
    float M = fmaxf(st.m[r], xor16(st.m[r]));
    M = fmaxf(M, xor32(M));
    const float w = st.m[r] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st.m[r] - M);
    float l = st.l[r] * w;
    l += xor16(l);
    l += xor32(l);
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      o[c] = st.o[r][c] * w;
      o[c] += xor16(o[c]);
      o[c] += xor32(o[c]);
    }
    if (rs == 0) {
      float* dst = sh + r * kPartialFloats + (wave * 16 + cn) * 10;
#pragma unroll
      for (int c = 0; c < 8; ++c) dst[c] = o[c];
      dst[8] = M;
      dst[9] = l;
    }
  }
  __syncthreads();
  // thread -> (head parity, channel): threads 0..127 take the even heads, 128..255 the odd ones
  const int ch = tid & 127, chunk = ch >> 3, e = ch & 7;
  for (int r = tid >> 7; r < NREP; r += 2) {
    const float* src = sh + r * kPartialFloats + chunk * 10;
    float M = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) M = fmaxf(M, src[wv * 160 + 8]);
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      const float ms = src[wv * 160 + 8];
      const float w = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - M);
      acc += w * src[wv * 160 + e];
      lsum += w * src[wv * 160 + 9];
    }
    const size_t ps = ((size_t)unit * NREP + r) * n_slots + slot;
    if (COHERENT) {  // read back by another workgroup of this kernel
      store_coherent(&po[ps * kD + ch], acc);
      if (ch == 0) {
        store_coherent(&pm[ps], M);
        store_coherent(&pl[ps], mark ? -(lsum + 1.f) : lsum);
      }
    } else {
      po[ps * kD + ch] = acc;
      if (ch == 0) {
        pm[ps] = M;
        pl[ps] = mark ? -(lsum + 1.f) : lsum;
      }
    }
  }
}

__device__ __forceinline__ float wave_allsum_f(float x) {
  x = row_allsum(x);
  x += xor16(x);
  x += xor32(x);
  return x;
}
__device__ __forceinline__ float wave_allmax_f(float x) {
  x = fmaxf(x, row_ror<8>(x));
  x = fmaxf(x, row_ror<4>(x));
  x = fmaxf(x, row_ror<2>(x));
  x = fmaxf(x, row_ror<1>(x));
  x = fmaxf(x, xor16(x));
  x = fmaxf(x, xor32(x));
  return x;
}

// Merge the partial slots [0, n_used) of all NREP query heads of a unit into out[NREP][128].  256 threads form
// four groups of 64 (thread k of a group owns channels 2k, 2k+1).  Each group folds the slots s = sub, sub + GPH,
// ... of one head with a running maximum, 32 or 40 slots per batch: their (m, l) sit one per lane and reach the other
// lanes as scalars, the independent 8-byte loads of o are in flight together, so that the round trips
// to memory overlap; with fewer than four heads several groups share a head and meet in LDS.
// A slot stored with a mark (l < 0, see store_partials) counts with its true l.
// sh: 4 * 130 floats.  Has barriers.
template <int NREP>
__device__ __forceinline__ void merge_heads(const float* __restrict__ po, const float* __restrict__ pm,
                                            const float* __restrict__ pl, int unit, int n_slots, int n_used,
                                            float* sh, float* __restrict__ out_unit) {
  constexpr int GPH = NREP == 1 ? 4 : (NREP == 2 ? 2 : 1);  // groups per head
  constexpr int BATCH = GPH == 1 ? 40 : 32;                 // slots per batch and group (a 128k context has 33)
  constexpr int HPP = 4 / GPH;                              // heads per pass
  const int tid = threadIdx.x, lane = tid & 63;
  const int k2 = lane * 2, g = tid >> 6;
#pragma unroll 1
  for (int h0 = 0; h0 < NREP; h0 += HPP) {
    const int h = h0 + g / GPH, sub = g % GPH;
    const bool head_ok = h < NREP;  // the same for the whole wavefront
    const size_t base = ((size_t)unit * NREP + (head_ok ? h : 0)) * n_slots;
    float M = -INFINITY, acc0 = 0.f, acc1 = 0.f, lsum = 0.f;
    for (int s0 = sub; s0 < n_used && head_ok; s0 += GPH * BATCH) {
      // (m, l) of the batch's slots live one per lane; every lane loads its two channels of all the slots
      const int sj = s0 + GPH * lane;
      const bool okj = lane < BATCH && sj < n_used;
      const float mj = okj ? load_coherent(&pm[base + sj]) : -INFINITY;
      float lj = okj ? load_coherent(&pl[base + sj]) : 0.f;
      unsigned long long os[BATCH];
#pragma unroll
      for (int k = 0; k < BATCH; ++k) {
        const int s = s0 + GPH * k;
        os[k] = load_coherent(reinterpret_cast<const unsigned long long*>(&po[(base + (s < n_used ? s : s0)) * kD + k2]));
      }
      lj = lj < 0.f ? -lj - 1.f : lj;
      const float mx = fmaxf(M, wave_allmax_f(mj));
      const float mref = mx == -INFINITY ? 0.f : mx;
      const float alpha = __builtin_amdgcn_exp2f(M - mref);
      const float wj = __builtin_amdgcn_exp2f(mj - mref);  // 0 for an empty slot
      acc0 *= alpha;
      acc1 *= alpha;
      lsum = lsum * alpha + wave_allsum_f(wj * lj);
#pragma unroll
      for (int k = 0; k < BATCH; ++k) {
        const float w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wj), k));
        acc0 += w * __uint_as_float((uint32_t)os[k]);
        acc1 += w * __uint_as_float((uint32_t)(os[k] >> 32));
      }
      M = mx;
    }
    __syncthreads();
    sh[g * 130 + k2] = acc0;
    sh[g * 130 + k2 + 1] = acc1;
    if (k2 == 0) {
      sh[g * 130 + 128] = lsum;
      sh[g * 130 + 129] = M;
    }
    __syncthreads();
    for (int o = tid; o < HPP * kD; o += 256) {
      const int hh = o / kD, c = o % kD;
      if (h0 + hh < NREP) {
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < GPH; ++j) mx = fmaxf(mx, sh[(hh * GPH + j) * 130 + 129]);
        const float mref = mx == -INFINITY ? 0.f : mx;
        float l = 0.f, a = 0.f;
#pragma unroll
        for (int j = 0; j < GPH; ++j) {
          const float w = __builtin_amdgcn_exp2f(sh[(hh * GPH + j) * 130 + 129] - mref);
          l += w * sh[(hh * GPH + j) * 130 + 128];
          a += w * sh[(hh * GPH + j) * 130 + c];
        }
        out_unit[(size_t)(h0 + hh) * kD + c] = l > 0.f ? a / l : 0.f;
      }
    }
  }
}

}  // namespace fier
