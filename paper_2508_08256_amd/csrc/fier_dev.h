// Device-side helpers shared by the Fier kernels (gfx950 only, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

// Optional time stamps for kernel tuning: `python -m paper_2508_08256_amd.build --prof` compiles the same sources
// with -DFIER_PROF_ENABLE plus fier_prof.hip (which defines the two arrays and the calls that read them) into
// libfier_prof.so.  The library proper is compiled without the flag and contains none of this.
#ifdef FIER_PROF_ENABLE
extern __device__ unsigned long long fier_prof_slots[64];
#define FIER_PROF(slot, cond)                                              \
  __builtin_amdgcn_sched_barrier(0);                                       \
  if ((cond) && threadIdx.x == 0) fier_prof_slots[slot] = wall_clock64();  \
  __builtin_amdgcn_sched_barrier(0);
// one time stamp per workgroup and point (the host reduces them)
extern __device__ unsigned long long fier_prof_wg[8][4096];
#define FIER_PROF_WG(point)                                                                  \
  if (threadIdx.x == 0 && blockIdx.y * gridDim.x + blockIdx.x < 4096)                        \
    fier_prof_wg[point][blockIdx.y * gridDim.x + blockIdx.x] = wall_clock64();
#else
#define FIER_PROF(slot, cond)
#define FIER_PROF_WG(point)
#endif

namespace fier {

constexpr int kD = 128;        // head_dim
constexpr int kG = 32;         // tokens per quantization group (Alg. 1 step 1)
constexpr int kPair = 64;      // tokens per packed "pair block" = one wavefront of tokens
constexpr int DT_F16 = 0;
constexpr int DT_BF16 = 1;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// ---- 16-bit storage formats <-> binary32 -------------------------------------------------------
template <int DT>
__device__ __forceinline__ float w2f(uint32_t w16) {
  if (DT == DT_F16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)w16);
  } else {
    return __uint_as_float(w16 << 16);
  }
}

// round to nearest even; the argument is finite and within the finite range of the format
template <int DT>
__device__ __forceinline__ uint32_t f2w(float x) {
  if (DT == DT_F16) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
  } else {
    uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
}

template <int DT>
__device__ __forceinline__ float lo16f(uint32_t pair) {
  if (DT == DT_F16) return (float)__builtin_bit_cast(half2_t, pair).x;
  return __uint_as_float(pair << 16);
}
template <int DT>
__device__ __forceinline__ float hi16f(uint32_t pair) {
  if (DT == DT_F16) return (float)__builtin_bit_cast(half2_t, pair).y;
  return __uint_as_float(pair & 0xffff0000u);
}

// two-element dot product with binary32 accumulate on the packed-16-bit pipeline
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
  if (DT == DT_F16) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc, false);
  } else {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc,
                                           false);
  }
}

// ---- cross-lane helpers ---------------------------------------------------------------------------
// DPP row rotate within each row of 16 lanes (dpp_ctrl 0x120 + n = row_ror:n)
template <int N>
__device__ __forceinline__ float row_ror(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + N, 0xf, 0xf, true));
}
// sum over the 16 lanes of a row, result in every lane of the row
__device__ __forceinline__ float row_allsum(float x) {
  x += row_ror<8>(x);
  x += row_ror<4>(x);
  x += row_ror<2>(x);
  x += row_ror<1>(x);
  return x;
}

__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

}  // namespace fier

namespace fier {

// order-preserving map binary32 -> uint32 (larger score <=> larger key); -0 and +0 share a key
__device__ __forceinline__ uint32_t score_key(float v) {
  v += 0.0f;
  uint32_t u = __float_as_uint(v);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

// bin of the equal-width histogram over [-R, R]; monotone non-decreasing in v, the same in every kernel.  The
// clamp is done in floating point (the maximum and minimum of a NaN and a number are the number), so the
// conversion to an integer always sees a value in [0, n_bins - 1]: with scale = 0 (R = 0: every score is zero)
// everything lands in bin 0.
__device__ __forceinline__ int sel_bin(float v, float R, float scale, int n_bins) {
  const float x = fminf(fmaxf((v + R) * scale, 0.0f), (float)(n_bins - 1));
  return (int)x;
}
// bins per unit of score for scores in [-R, R]; 0 when the range is empty
__device__ __forceinline__ float sel_scale(float R, int n_bins) { return R > 0.0f ? (float)n_bins / (R + R) : 0.0f; }

// Inclusive prefix sum over the 64 lanes with DPP (row shifts inside each row of 16 lanes, then the last lane of
// a row broadcast into the following rows): six dependent ALU ops instead of six LDS-crossbar shuffles.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add_u32(uint32_t v) {
  return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int /*lane*/) {
  v = dpp_add_u32<0x111, 0xf>(v);  // row_shr:1
  v = dpp_add_u32<0x112, 0xf>(v);  // row_shr:2
  v = dpp_add_u32<0x114, 0xf>(v);  // row_shr:4
  v = dpp_add_u32<0x118, 0xf>(v);  // row_shr:8
  v = dpp_add_u32<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_add_u32<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
  return v;
}
// Sum over the 64 lanes, the same value in every lane.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan_u32(v, 0), 63);
}

// Exclusive scan over the threads of a workgroup of NW wavefronts (thread order) and the total.
// tmp: NW words of LDS.  Contains two barriers.
template <int NW>
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, uint32_t* tmp, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(v, lane);
  __syncthreads();
  if (lane == 63) tmp[wave] = incl;
  __syncthreads();
  const uint32_t wsum = lane < NW ? tmp[lane] : 0;
  const uint32_t wincl = wave_incl_scan_u32(wsum, lane);
  const int w = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t wave_off =
      (uint32_t)__builtin_amdgcn_readlane((int)wincl, w) - (uint32_t)__builtin_amdgcn_readlane((int)wsum, w);
  total = (uint32_t)__builtin_amdgcn_readlane((int)wincl, NW - 1);
  return wave_off + incl - v;
}

// ---- publishing results to another workgroup of the same kernel -------------------------------------------
// The L2 caches of the eight XCDs are not coherent with each other.  A device-scope fence (__threadfence)
// writes back / invalidates a whole L2 and costs tens of microseconds when a thousand workgroups do it, so
// the few words one workgroup hands to another are instead written with device-scope atomic stores (write
// through to memory) and read with device-scope atomic loads; the arrival counter is a device-scope atomic.
// Before the arrival is counted every wave waits for the acknowledgement of its own stores (an explicit
// s_waitcnt: the workgroup-scope fence of __syncthreads does not wait for global stores, since the waves of a
// workgroup share one L1), and the barrier then orders all of them before the counting wave's atomic.
__device__ __forceinline__ void store_coherent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t load_coherent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_coherent(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Arrival at a unit's counter: adds `inc` and returns, in every thread, the value the counter held before.
// Everything the workgroups that arrived earlier published with store_coherent / atomics before arriving can then be
// read with load_coherent.  Nobody waits for anybody.  flag: one word of LDS.
__device__ __forceinline__ uint32_t arrive_add(uint32_t* counter, uint32_t inc, uint32_t* flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's stores and atomics have been acknowledged
  __syncthreads();                                  // ... and so have those of the other waves
  if (threadIdx.x == 0) *flag = __hip_atomic_fetch_add(counter, inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const uint32_t before = *flag;
  // reader side: nothing the last arriver loads afterwards may be moved above the counter's return by the compiler
  // (the hardware issues a wave's memory operations in program order, and load_coherent never hits a stale line)
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  asm volatile("" ::: "memory");
  return before;
}
// "Last arriver": true in every thread of exactly one workgroup per counter, the one whose increment brings it to
// `expected`.
__device__ __forceinline__ bool last_arriver(uint32_t* counter, uint32_t expected, uint32_t* flag) {
  return arrive_add(counter, 1u, flag) == expected - 1;
}

// A load with the streaming hint, for data that is read once (K / V rows of a large gather, the packed key codes).
__device__ __forceinline__ uint32_t load_stream(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
  const u4_t v = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

}  // namespace fier
