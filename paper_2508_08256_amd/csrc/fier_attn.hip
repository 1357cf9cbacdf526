// Exact attention over a selected subset of K/V rows (Alg. 1 step 4), and over the whole cache when no
// index list is given (the decode attention of Sec. 3.1).
//
// Split-K: workgroup (split, unit) owns `rows_per_wg` consecutive entries of the unit's selection and
// produces one partial (m, l, o[128]) per query head; a second kernel merges the partials with the
// usual running-max rescale.  Inside a workgroup a row of 16 lanes owns one K/V row at a time: lane n of
// the row loads channels 8n..8n+7 as one 16-byte request, so a wavefront fetches 4 whole 256-byte rows
// per load instruction and 4 such loads (16 rows) of K and of V are in flight per iteration.  The
// q.k products use the packed 16-bit dot instructions with binary32 accumulation, are reduced over the
// 16 lanes with DPP rotates, and softmax / PV run in binary32 with exp2.
#include "fier_dev.h"
#include "fier_kernels.h"

namespace fier {

constexpr int kAttnUnroll = 4;                  // rows per 16-lane row per iteration
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

// Attend over entries [start, end) of a row list; row_of(j) gives the row of entry j in the K / V arrays (the
// callers map a token to its row: contiguous, or through the block table).  The workgroup's
// 16 lane rows (4 waves x 4) take entries round-robin in batches of kAttnUnroll.
template <int DT, int NREP, class RowOf>
__device__ __forceinline__ void attend_rows(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                            const uint4 (&qr)[NREP], RowOf row_of, int start, int end,
                                            float scale_log2e, AttnState<NREP>& st) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rs = lane >> 4, cn = lane & 15;
  for (int i0 = start + wave * (4 * kAttnUnroll); i0 < end; i0 += kRowsPerIter) {
    uint4 kk[kAttnUnroll], vv[kAttnUnroll];
    bool valid[kAttnUnroll];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int j = i0 + u * 4 + rs;
      valid[u] = j < end;
      const size_t ro = row_of(valid[u] ? j : start) * (kD / 8) + cn;
      kk[u] = K[ro];
      vv[u] = V[ro];
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
// q_unit: the unit's NREP query rows; sh: kAttnMfmaLds floats of LDS.
template <int DT, int NREP, class RowOf>
__device__ __forceinline__ void attend_rows_mfma(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                 const uint4* __restrict__ q_unit, RowOf row_of, int start, int end,
                                                 float scale_log2e, AttnState<NREP>& st, float* sh) {
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
  for (int j0 = start + wave * 16; j0 < end; j0 += 64) {
    // K rows in the matrix view (token j0 + n), V rows in the row-owner view (tokens j0 + 4u + kq, channels 8n..8n+7)
    const int jk = j0 + n;
    const bool valid = jk < end;
    uint4 kk[4], vv[4];
    const size_t rk = row_of(valid ? jk : start) * (kD / 8);
#pragma unroll
    for (int c = 0; c < 4; ++c) kk[c] = K[rk + 4 * c + kq];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int jv = j0 + 4 * u + kq;
      vv[u] = V[row_of(jv < end ? jv : start) * (kD / 8) + n];
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
template <int NREP, bool COHERENT>
__device__ __forceinline__ void store_partials(const AttnState<NREP>& st, float* sh, int unit, int n_slots, int slot,
                                               float* __restrict__ po, float* __restrict__ pm,
                                               float* __restrict__ pl) {
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
        store_coherent(&pl[ps], lsum);
      }
    } else {
      po[ps * kD + ch] = acc;
      if (ch == 0) {
        pm[ps] = M;
        pl[ps] = lsum;
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
      const float lj = okj ? load_coherent(&pl[base + sj]) : 0.f;
      unsigned long long os[BATCH];
#pragma unroll
      for (int k = 0; k < BATCH; ++k) {
        const int s = s0 + GPH * k;
        os[k] = load_coherent(reinterpret_cast<const unsigned long long*>(&po[(base + (s < n_used ? s : s0)) * kD + k2]));
      }
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

// Stand-alone attention (fier_sparse_attn: rows from an index list; fier_dense_attn: all rows).  grid (n_splits,
// units), block 256: a workgroup attends over rows_per_wg entries and stores one partial per query head; the unit's
// last workgroup merges the partials of the splits in use (arrival counter in the unit's control block).
template <int DT, int NREP>
__global__ __launch_bounds__(256) void attn_split_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                         const uint4* __restrict__ q, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ seq_lens, int extra,
                                                         int max_budget, int rows_per_wg, int n_splits,
                                                         float scale_log2e, float* __restrict__ po,
                                                         float* __restrict__ pm, float* __restrict__ pl,
                                                         UnitCtl* __restrict__ ctl, float* __restrict__ out,
                                                         int n_kv_heads, int max_ctx, int unit_major, KvLayout lay) {
  __shared__ float sh_o[NREP * kPartialFloats];
  __shared__ uint32_t flag;

  const int cn = threadIdx.x & 15;
  const int unit = unit_major ? blockIdx.x : blockIdx.y, split = unit_major ? blockIdx.y : blockIdx.x;
  const int b = unit / n_kv_heads;
  int n;
  if (idx) {
    n = count[unit];
    n = n > max_budget ? max_budget : n;
  } else {
    n = seq_lens[b] + extra;
    n = n > max_ctx ? max_ctx : n;
  }
  const int start = split * rows_per_wg;
  if (n <= 0 && split == 0) {  // nothing to attend over: zeros
    for (int o = threadIdx.x; o < NREP * kD; o += 256) out[(size_t)unit * NREP * kD + o] = 0.f;
    return;
  }
  if (start >= n) return;
  const int end = n < start + rows_per_wg ? n : start + rows_per_wg;
  const int32_t* __restrict__ sel = idx ? idx + (size_t)unit * max_budget : nullptr;
  const KvRows kv = lay.rows_of(unit);
  // whole-cache attention over paged rows: the block numbers of this workgroup's rows wait in LDS
  __shared__ int32_t lblk[kAttnRowsDenseMax / 64];
  const bool window = !sel && kv.blocks != nullptr;
  if (window) {
    const int bi = (start >> kv.shift) + (int)threadIdx.x;
    if (threadIdx.x < kAttnRowsDenseMax / 64) lblk[threadIdx.x] = bi < lay.blocks_per_seq ? kv.blocks[bi] : 0;
    __syncthreads();
  }
  const int first_block = start >> kv.shift;
  auto row_sel = [&](int j) {
    int t = sel[j];
    t = (t < 0 || t >= max_ctx) ? 0 : t;
    return kv.row(t);
  };
  auto row_all = [&](int j) {
    return window ? (size_t)lblk[(j >> kv.shift) - first_block] * kv.block_stride + kv.base + (size_t)(j & kv.mask)
                  : kv.base + (size_t)j;
  };

  uint4 qr[NREP];
#pragma unroll
  for (int r = 0; r < NREP; ++r) qr[r] = q[((size_t)unit * NREP + r) * (kD / 8) + cn];

  AttnState<NREP> st;
  st.init();
  if constexpr (NREP >= 3) {
    const uint4* q_unit = q + (size_t)unit * NREP * (kD / 8);
    if (sel)
      attend_rows_mfma<DT, NREP>(K, V, q_unit, row_sel, start, end, scale_log2e, st, sh_o);
    else
      attend_rows_mfma<DT, NREP>(K, V, q_unit, row_all, start, end, scale_log2e, st, sh_o);
  } else {
    if (sel)
      attend_rows<DT, NREP>(K, V, qr, row_sel, start, end, scale_log2e, st);
    else
      attend_rows<DT, NREP>(K, V, qr, row_all, start, end, scale_log2e, st);
  }
  store_partials<NREP, true>(st, sh_o, unit, n_splits, split, po, pm, pl);
  // the unit's last workgroup merges the partials of the splits in use
  const int used = (n + rows_per_wg - 1) / rows_per_wg;
  if (!last_arriver(&ctl[unit].arrive[0], (uint32_t)used, &flag)) return;
  merge_heads<NREP>(po, pm, pl, unit, n_splits, used, sh_o, out + (size_t)unit * NREP * kD);
  if (threadIdx.x == 0) ctl[unit].arrive[0] = 0;
}

// Third kernel of the fused decode step.  grid (ceil(n_ranges / RPW), units), block 256: the workgroup owns RPW
// consecutive 1024-token ranges of its unit (RPW is chosen by the host so that a workgroup has on the order of a
// hundred selected rows).  It re-reads their scores, applies the exact selection rule fixed by the threshold
// kernel, writes its part of the ascending index list, and attends over its selected rows straight from an LDS
// list -- the index list never has to be read back.  The unit's last workgroup merges the partials.
template <int DT, int NREP, int RPW>
__global__ __launch_bounds__(256) void select_attend_kernel(
    const float* __restrict__ scores, UnitCtl* __restrict__ ctl, const uint32_t* __restrict__ range_off,
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint4* __restrict__ q,
    const int32_t* __restrict__ seq_lens, int extra, int max_budget, float scale_log2e, float* __restrict__ po,
    float* __restrict__ pm, float* __restrict__ pl, int32_t* __restrict__ idx_out, float* __restrict__ out,
    float* __restrict__ kabsmax, const float* __restrict__ newmax, int n_ranges, int n_kv_heads, int max_ctx,
    int order, int wgs_per_unit, KvLayout lay) {
  __shared__ float sh_o[NREP * kPartialFloats > 4 * 130 ? NREP * kPartialFloats : 4 * 130];
  __shared__ uint16_t rows[kRangeTokens * RPW];  // selected tokens, relative to the workgroup's first token
  __shared__ uint32_t scan_tmp[4];
  __shared__ uint32_t flag;
  __shared__ int32_t lblk[RPW * kRangeTokens / 64];  // paged rows: block numbers of this workgroup's tokens

  const int tid = threadIdx.x;
  const int cn = tid & 15;
  // order: 0 = grid (workgroups, units); 1 = grid (units, workgroups); 2 = one-dimensional, groups of 8 units, a
  // group's workgroups together and unit % 8 fastest (see the launcher)
  int unit, wg;
  if (order == 2) {
    const int id = blockIdx.x;
    const int g = id / (8 * wgs_per_unit);
    const int rem = id - g * 8 * wgs_per_unit;
    wg = rem >> 3;
    unit = 8 * g + (rem & 7);
  } else {
    unit = order ? blockIdx.x : blockIdx.y;
    wg = order ? blockIdx.y : blockIdx.x;
  }
  const int b = unit / n_kv_heads;
  int n = seq_lens[b] + extra;
  n = n < 0 ? 0 : (n > max_ctx ? max_ctx : n);
  const int tok0 = wg * RPW * kRangeTokens;
  if (tok0 >= n && wg != 0) return;
  FIER_PROF(20, unit == 0 && wg == 3)
  FIER_PROF_WG(5)
  const KvRows kv = lay.rows_of(unit);
  if (kv.blocks && tid < RPW * kRangeTokens / 64) {  // in flight during the selection; barriers follow
    const int bi = (tok0 >> kv.shift) + tid;
    lblk[tid] = bi < lay.blocks_per_seq ? kv.blocks[bi] : 0;
  }
  UnitCtl* __restrict__ c = &ctl[unit];
  const int tbin = c->tbin;
  const float R = c->R, hscale = c->scale;
  const uint32_t T = c->T;
  const int32_t idxT = c->idxT;
  const int n_slots = wgs_per_unit;

  // ---- exact selection inside this workgroup's ranges, in token order ---------------------------------------
  float4 v[RPW];
  uint32_t off[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    v[rr] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n) v[rr] = *reinterpret_cast<const float4*>(scores + (size_t)unit * max_ctx + i);
    const int r = wg * RPW + rr;
    off[rr] = r < n_ranges ? range_off[(size_t)unit * n_ranges + r] : 0;
  }
  // selection flags of the thread's 4 tokens in each range, and their count
  uint32_t selm[RPW], cnt[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int i = tok0 + rr * kRangeTokens + 4 * tid;
    const float vv[4] = {v[rr].x, v[rr].y, v[rr].z, v[rr].w};
    selm[rr] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int bin = sel_bin(vv[j], R, hscale, kSelBins);
      const uint32_t key = score_key(vv[j]);
      const bool sel = i + j < n && (bin > tbin || (bin == tbin && (key > T || (key == T && i + j <= idxT))));
      selm[rr] |= sel ? 1u << j : 0u;
    }
    cnt[rr] = __builtin_popcount(selm[rr]);
  }
  // positions in token order: one workgroup scan serves two ranges (16 bits each: a range holds <= 1024 tokens)
  uint32_t n_sel_total = 0;
#pragma unroll
  for (int r2 = 0; r2 < RPW; r2 += 2) {
    const uint32_t packed = cnt[r2] | (r2 + 1 < RPW ? cnt[r2 + 1 < RPW ? r2 + 1 : r2] << 16 : 0u);
    uint32_t total;
    const uint32_t before = block_excl_scan_u32<4>(packed, scan_tmp, total);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int rr = r2 + h;
      if (rr < RPW) {
        const int i = tok0 + rr * kRangeTokens + 4 * tid;
        uint32_t pos = (before >> (16 * h)) & 0xffffu;
        const uint32_t n_sel = (total >> (16 * h)) & 0xffffu;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (selm[rr] >> j & 1u) {
            rows[n_sel_total + pos] = (uint16_t)(i + j - tok0);
            if (idx_out && off[rr] + pos < (uint32_t)max_budget)
              idx_out[(size_t)unit * max_budget + off[rr] + pos] = i + j;
            ++pos;
          }
        n_sel_total += n_sel;
      }
    }
  }
  __syncthreads();
  FIER_PROF(21, unit == 0 && wg == 3)

  // ---- attention over the selected rows of these ranges --------------------------------------------------------
  uint4 qr[NREP];
#pragma unroll
  for (int h = 0; h < NREP; ++h) qr[h] = q[((size_t)unit * NREP + h) * (kD / 8) + cn];
  AttnState<NREP> st;
  st.init();
  const int first_block = tok0 >> kv.shift;
  auto row_of = [&](int j) {
    const int t = tok0 + (int)rows[j];
    return kv.blocks ? (size_t)lblk[(t >> kv.shift) - first_block] * kv.block_stride + kv.base + (size_t)(t & kv.mask)
                     : kv.base + (size_t)t;
  };
  if constexpr (NREP >= 3)
    attend_rows_mfma<DT, NREP>(K, V, q + (size_t)unit * NREP * (kD / 8), row_of, 0, (int)n_sel_total, scale_log2e, st,
                               sh_o);
  else
    attend_rows<DT, NREP>(K, V, qr, row_of, 0, (int)n_sel_total, scale_log2e, st);
  FIER_PROF(22, unit == 0 && wg == 3)
  store_partials<NREP, true>(st, sh_o, unit, n_slots, wg, po, pm, pl);
  FIER_PROF(23, unit == 0 && wg == 3)
  FIER_PROF_WG(6)

  const int n_wgs = (n + RPW * kRangeTokens - 1) / (RPW * kRangeTokens);  // workgroups of this unit in use
  if (!last_arriver(&c->arrive[2], n_wgs > 0 ? (uint32_t)n_wgs : 1u, &flag)) return;
  FIER_PROF(24, unit == 0)
  // ---- the unit's last workgroup merges the partials of all workgroups --------------------------------------
  merge_heads<NREP>(po, pm, pl, unit, n_slots, n_wgs, sh_o, out + (size_t)unit * NREP * kD);
  if (tid == 0) c->arrive[2] = 0;
  FIER_PROF(25, unit == 0)
  FIER_PROF_WG(7)
  // the step appended a row: fold the bound of its re-quantized group into the unit's per-channel bound
  if (extra && seq_lens[b] < max_ctx && tid < kD) {
    float* slot = kabsmax + (size_t)unit * kD + tid;
    const float a = newmax[(size_t)unit * kD + tid];
    if (a > *slot) *slot = a;
  }
}

template <int DT>
static hipError_t launch_attn_dt(KvLayout lay, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                                 const int32_t* count, const int32_t* seq_lens, int extra, int max_budget,
                                 int rows_per_wg, int n_splits, float sm_scale, float* po, float* pm, float* pl,
                                 UnitCtl* ctl, float* out, int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  // dispatch order as in the select + attend kernel, for gathers; whole-cache attention streams and gains nothing
  const int unit_major = idx != nullptr && (long)units * n_splits <= 2 * 256L * (n_rep >= 3 ? 4 : 7) ? 1 : 0;
  dim3 grid = unit_major ? dim3(units, n_splits) : dim3(n_splits, units);
  const float sl2 = sm_scale * 1.4426950408889634f;
  if (!idx && rows_per_wg > kAttnRowsDenseMax) return hipErrorInvalidValue;  // the kernel's block-number window
#define FIER_ATTN_CASE(R)                                                                                          \
  case R:                                                                                                          \
    attn_split_kernel<DT, R><<<grid, 256, 0, st>>>((const uint4*)K, (const uint4*)V, (const uint4*)q, idx, count,  \
                                                   seq_lens, extra, max_budget, rows_per_wg, n_splits, sl2, po, pm, \
                                                   pl, ctl, out, n_kv_heads, max_ctx, unit_major, lay);            \
    break;
  switch (n_rep) {
    FIER_ATTN_CASE(1)
    FIER_ATTN_CASE(2)
    FIER_ATTN_CASE(3)
    FIER_ATTN_CASE(4)
    FIER_ATTN_CASE(5)
    FIER_ATTN_CASE(6)
    FIER_ATTN_CASE(7)
    FIER_ATTN_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_ATTN_CASE
  return hipGetLastError();
}

template <int DT, int RPW>
static hipError_t launch_select_attend_dt(KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                          const void* q, const int32_t* seq_lens, int extra, int max_budget,
                                          float sm_scale, int32_t* idx_out, float* out, float* kabsmax, int units,
                                          int n_kv_heads, int max_ctx, hipStream_t st) {
  const int n_ranges = (max_ctx + kRangeTokens - 1) / kRangeTokens;
  const int n_wgs = (n_ranges + RPW - 1) / RPW;
  // Dispatch order.  Workgroups go round-robin to the 8 XCDs in the order of their linear index; when a unit's
  // workgroups all run on one XCD, its scores, offsets, partials and arrival counter stay in that XCD's L2.
  //   1: units fastest (a multiple of 8 units puts unit u on XCD u % 8), for grids of at most about two resident
  //      rounds (256 CUs x 4 workgroups of this kernel for 3+ query heads per kv head, x 7 otherwise):
  //      20.8 -> 19.6 us at config 2, 29.4 -> 26.5 us at config 3 against order 0;
  //   2: longer grids with a multiple of 8 units: groups of 8 units one after the other, inside a group the
  //      workgroups in range order and unit % 8 fastest -- the same XCD assignment, but a sequence's ranges stay
  //      together in time (the ragged 128-unit batch: 69.9 -> 62.9 us against order 0; order 1 there: 75.5 us);
  //   0: ranges fastest, otherwise.
  const int order = (long)units * n_wgs <= 2 * 256L * (n_rep >= 3 ? 4 : 7) ? 1 : (units % 8 == 0 ? 2 : 0);
  dim3 grid = order == 2 ? dim3((unsigned)units * (unsigned)n_wgs) : (order ? dim3(units, n_wgs) : dim3(n_wgs, units));
  const float sl2 = sm_scale * 1.4426950408889634f;
#define FIER_SA_CASE(R)                                                                                            \
  case R:                                                                                                          \
    select_attend_kernel<DT, R, RPW><<<grid, 256, 0, st>>>(                                                        \
        sb.scores, sb.ctl, sb.range_cnt, (const uint4*)K, (const uint4*)V, (const uint4*)q, seq_lens, extra,       \
        max_budget, sl2, sb.po, sb.pm, sb.pl, idx_out, out, kabsmax, sb.newmax, n_ranges, n_kv_heads, max_ctx,     \
        order, n_wgs, lay);                                                                                        \
    break;
  switch (n_rep) {
    FIER_SA_CASE(1)
    FIER_SA_CASE(2)
    FIER_SA_CASE(3)
    FIER_SA_CASE(4)
    FIER_SA_CASE(5)
    FIER_SA_CASE(6)
    FIER_SA_CASE(7)
    FIER_SA_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef FIER_SA_CASE
  return hipGetLastError();
}

int select_attend_ranges_per_wg(int max_budget, int max_ctx) {
  // about a hundred selected rows per workgroup: rows per 1024-token range = 1024 * budget / context
  const double per_range = 1024.0 * (double)max_budget / (double)max_ctx;
  int rpw = 1;
  while (rpw < 8 && per_range * rpw < 96.0) rpw *= 2;
  return rpw;
}

hipError_t launch_select_attend(int dtype, KvLayout lay, int n_rep, const StepBuffers& sb, const void* K, const void* V,
                                const void* q, const int32_t* seq_lens, int extra, int max_budget, float sm_scale,
                                int32_t* idx_out, float* out, float* kabsmax, int units, int n_kv_heads, int max_ctx,
                                hipStream_t st) {
#define FIER_SA_RPW(DT, RPW)                                                                                        \
  return launch_select_attend_dt<DT, RPW>(lay, n_rep, sb, K, V, q, seq_lens, extra, max_budget, sm_scale, idx_out, out, \
                                          kabsmax, units, n_kv_heads, max_ctx, st)
  const int rpw = select_attend_ranges_per_wg(max_budget, max_ctx);
  if (dtype == DT_F16) {
    if (rpw == 1) FIER_SA_RPW(DT_F16, 1);
    if (rpw == 2) FIER_SA_RPW(DT_F16, 2);
    if (rpw == 4) FIER_SA_RPW(DT_F16, 4);
    FIER_SA_RPW(DT_F16, 8);
  }
  if (rpw == 1) FIER_SA_RPW(DT_BF16, 1);
  if (rpw == 2) FIER_SA_RPW(DT_BF16, 2);
  if (rpw == 4) FIER_SA_RPW(DT_BF16, 4);
  FIER_SA_RPW(DT_BF16, 8);
#undef FIER_SA_RPW
}

hipError_t launch_attn(int dtype, KvLayout lay, int n_rep, const void* K, const void* V, const void* q, const int32_t* idx,
                       const int32_t* count, const int32_t* seq_lens, int extra, int max_budget, int rows_per_wg,
                       int n_splits, float sm_scale, float* po, float* pm, float* pl, UnitCtl* ctl, float* out,
                       int units, int n_kv_heads, int max_ctx, hipStream_t st) {
  if (dtype == DT_F16)
    return launch_attn_dt<DT_F16>(lay, n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                                  sm_scale, po, pm, pl, ctl, out, units, n_kv_heads, max_ctx, st);
  return launch_attn_dt<DT_BF16>(lay, n_rep, K, V, q, idx, count, seq_lens, extra, max_budget, rows_per_wg, n_splits,
                                 sm_scale, po, pm, pl, ctl, out, units, n_kv_heads, max_ctx, st);
}

}  // namespace fier
