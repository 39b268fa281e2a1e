// Rotary-embedding arithmetic shared by the kernels that rotate new tokens: fp64 rotation of a
// pair, rounded once to bf16, so that every kernel produces the same bits for the same input.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace efim {

__device__ __forceinline__ double bf16_bits_to_f64(uint32_t bits16) {
  return (double)__uint_as_float(bits16 << 16);
}

// fp64 -> bf16, round to nearest even, with a single rounding.  The conversion goes through
// fp32; the only case where the detour could round twice is an inexact fp32 result sitting
// exactly on a bf16 midpoint, which is nudged to the side the exact value lies on.
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double x) {
  float f = (float)x;
  uint32_t u = __float_as_uint(f);
  if ((u & 0xFFFFu) == 0x8000u) {
    double back = (double)f;
    if (back != x) u = (fabs(x) > fabs(back)) ? u + 1u : u - 1u;
  }
  // round to nearest even on the upper 16 bits (NaN stays NaN: quiet bit is in the upper half)
  uint32_t lsb = (u >> 16) & 1u;
  if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + lsb;
  return u >> 16;
}

// (x1, x2) rotated by the angle whose cosine and sine are c and s; products and sums are
// separate fp64 operations (no fused multiply-add), then one rounding to bf16 each.
__device__ __forceinline__ void rotate_pair_bf16(uint32_t x1_bits, uint32_t x2_bits, double c, double s,
                                                 uint32_t* y1_bits, uint32_t* y2_bits) {
#pragma clang fp contract(off)
  const double x1 = bf16_bits_to_f64(x1_bits), x2 = bf16_bits_to_f64(x2_bits);
  *y1_bits = f64_to_bf16_bits(x1 * c - x2 * s);
  *y2_bits = f64_to_bf16_bits(x2 * c + x1 * s);
}

}  // namespace efim
