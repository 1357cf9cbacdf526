// Device-side helpers shared by the Fier kernels (gfx950 only, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
