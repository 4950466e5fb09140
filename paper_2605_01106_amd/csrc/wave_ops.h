// Wavefront-level helpers shared by the kernels: sums over the 64 lanes through DPP row
// butterflies, the ordered key of the LM-head argmax, and the bfloat16 rounding of stored values.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hh {

// v of lane l combined with the lane that a DPP control selects (row_shr, quad_perm, row_bcast ...)
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// sum over each row of 16 lanes, left in every lane of the row
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return v;
}
// sum over the 64 lanes (the four row totals added in row order), uniform result
__device__ __forceinline__ float wave_sum64(float v) {
  v = row16_sum(v);
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

// Key whose unsigned order is (larger value first, then lower index): the maximum over keys is the
// argmax with the lowest index among equal values.
__device__ __forceinline__ unsigned long long argmax_key(float v, int n) {
  uint32_t u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (static_cast<unsigned long long>(u) << 32) | static_cast<unsigned long long>(0xFFFFFFFFu - (uint32_t)n);
}

// float32 -> bfloat16 bits, round to nearest even (the rounding of every value stored as bf16)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

}  // namespace hh
