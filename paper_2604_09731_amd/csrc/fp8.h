// E4M3 (OCP 8-bit floating point, finite-only variant: bias 7, no infinities, S.1111.111 = NaN,
// largest finite value 448) <-> binary32, in software: the cache writers must round and saturate
// the same way on every path, and decoding is exact anyway.
#ifndef SMART_FP8_H_
#define SMART_FP8_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace smart {

__device__ inline float fp8_e4m3_to_float(uint8_t c) {
  const uint32_t sign = (uint32_t)(c & 0x80u) << 24;
  const uint32_t e = (c >> 3) & 0xFu, m = c & 7u;
  if (e == 0) return __uint_as_float(sign | __float_as_uint((float)m * 0.001953125f));  // m * 2^-9
  if (e == 15 && m == 7) return __uint_as_float(sign | 0x7FC00000u);
  return __uint_as_float(sign | ((e + 120u) << 23) | (m << 20));
}

// Round to nearest, ties to the even mantissa; anything beyond 448 (infinities included) becomes
// +-448; NaN becomes 0x7F.
__device__ inline uint8_t float_to_fp8_e4m3(float x) {
  const uint32_t u = __float_as_uint(x);
  const uint32_t sign = (u >> 24) & 0x80u;
  const uint32_t a = u & 0x7FFFFFFFu;
  if (a > 0x7F800000u) return 0x7F;
  const float f = __uint_as_float(a);
  if (f >= 448.f) return (uint8_t)(sign | 0x7Eu);
  if (f < 0.015625f) return (uint8_t)(sign | (uint32_t)rintf(f * 512.f));  // multiples of 2^-9; 8 is the smallest normal
  uint32_t r = (a + 0x7FFFFu + ((a >> 20) & 1u)) >> 20;  // exponent and three mantissa bits, rounded
  r -= 120u << 3;
  return (uint8_t)(sign | (r > 0x7Eu ? 0x7Eu : r));
}

}  // namespace smart
#endif
