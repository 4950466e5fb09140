// Exact three-term bf16 split of a float32 value for the matrix-core kernels:
// x = t0 + t1 + t2 with t0 = bf16(x), t1 = bf16(x - t0), t2 = bf16(x - t0 - t1) (8 + 8 + 8
// mantissa bits; the two subtractions are exact).  The roundings use the hardware conversion
// (v_cvt_pk_bf16_f32, round to nearest even).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hh {

__device__ __forceinline__ uint32_t bf16_bits_hw(float f) {
  const __bf16 b = static_cast<__bf16>(f);
  return static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(&b));
}

__device__ __forceinline__ void split3_bf16(float x, uint32_t& t0, uint32_t& t1, uint32_t& t2) {
  t0 = bf16_bits_hw(x);
  const float r1 = x - __uint_as_float(t0 << 16);
  t1 = bf16_bits_hw(r1);
  const float r2 = r1 - __uint_as_float(t1 << 16);
  t2 = bf16_bits_hw(r2);
}

// The same split for two values at once; word k holds term k of a (low half) and of b (high half).
typedef float split_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 split_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pair_hw(float a, float b) {
  const split_f32x2 v = {a, b};
  const split_bf16x2 r = __builtin_convertvector(v, split_bf16x2);
  return *reinterpret_cast<const uint32_t*>(&r);
}
__device__ __forceinline__ void split3_bf16_pair(float a, float b, uint32_t& w0, uint32_t& w1, uint32_t& w2) {
  w0 = bf16_pair_hw(a, b);
  const float ra = a - __uint_as_float(w0 << 16), rb = b - __uint_as_float(w0 & 0xffff0000u);
  w1 = bf16_pair_hw(ra, rb);
  const float sa = ra - __uint_as_float(w1 << 16), sb = rb - __uint_as_float(w1 & 0xffff0000u);
  w2 = bf16_pair_hw(sa, sb);
}

// Two terms only: a + b's leading 16 mantissa bits (relative error 2^-17).
__device__ __forceinline__ void split2_bf16_pair(float a, float b, uint32_t& w0, uint32_t& w1) {
  w0 = bf16_pair_hw(a, b);
  w1 = bf16_pair_hw(a - __uint_as_float(w0 << 16), b - __uint_as_float(w0 & 0xffff0000u));
}

}  // namespace hh
