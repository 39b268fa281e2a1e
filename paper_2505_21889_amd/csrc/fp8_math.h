// 8-bit floating point (OCP FP8 E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
// infinities, largest finite value 448) as used for the 8-bit KV cache.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace efim {

// binary32 -> E4M3 code: round to nearest, ties to the even code; magnitudes of 448 and above
// saturate to +-448; NaN gives the NaN code.  Integer arithmetic on the bit pattern, so the
// result does not depend on any conversion instruction's mode bits.
__device__ __forceinline__ uint32_t f32_to_e4m3(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t sign = (u >> 24) & 0x80u;
  const uint32_t a = u & 0x7FFFFFFFu;
  if (a > 0x7F800000u) return 0x7Fu;                 // NaN
  if (a >= 0x43E00000u) return sign | 0x7Eu;         // |f| >= 448
  if (a >= 0x3C800000u) {                            // |f| >= 2^-6: normal E4M3 range
    // keep 3 mantissa bits: add half of the dropped part (less one when the kept part is even)
    const uint32_t r = (a + 0x7FFFFu + ((a >> 20) & 1u)) >> 20;  // (biased exponent << 3) | mantissa
    return sign | (r - ((127u - 7u) << 3));
  }
  // below the smallest normal the codes are the integers m = |f| * 2^9 (m == 8 is 2^-6 itself)
  return sign | (uint32_t)__builtin_rintf(__builtin_fabsf(f) * 512.f);
}

// Code of a bf16 value (bit pattern) under a per-tensor scale: the quotient is the binary32
// division, correctly rounded.
__device__ __forceinline__ uint32_t bf16_bits_to_e4m3(uint32_t bits16, float scale) {
  return f32_to_e4m3(__fdiv_rn(__uint_as_float(bits16 << 16), scale));
}

}  // namespace efim
