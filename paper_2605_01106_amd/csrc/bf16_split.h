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

}  // namespace hh
