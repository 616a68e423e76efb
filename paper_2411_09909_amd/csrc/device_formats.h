// Device-side decoding of the 8-bit shared scales and the FP4 E2M1 element codes (Sec. 2.1, Sec. 4.2 Eq. 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace amx {

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// Value of a scale byte as an exact float. E5M2 is the upper byte of an IEEE half (subnormals included); E4M3 has
// exponent bias 7 and subnormals m * 2^-9 (the sign bit of either FP8 byte is never set by the cast and is ignored);
// E8M0 is a bare exponent with bias 127 (byte 0 = 2^-127, an FP32 subnormal).
template <int SCALE_KIND>
__device__ __forceinline__ float scale_value(uint32_t byte) {
  if constexpr (SCALE_KIND == kScaleE5M2) {
    // the byte is the upper byte of an IEEE half: the half -> float conversion is exact, subnormals included
    return (float)__builtin_bit_cast(_Float16, (uint16_t)((byte & 0x7Fu) << 8));
  } else if constexpr (SCALE_KIND == kScaleE4M3) {
    // 0eeeemmm << 7 read as a half is (1 + m/8) * 2^(e - 15), or (m/8) * 2^-14 for e = 0: 2^8 times that is the value
    return (float)__builtin_bit_cast(_Float16, (uint16_t)((byte & 0x7Fu) << 7)) * 256.0f;
  } else {
    return byte == 0 ? u2f(0x00400000u) : u2f(byte << 23);  // 2^(byte-127)
  }
}

// 2 * |E2M1 value| for the 3-bit magnitude code: {0,1,2,3,4,6,8,12}, packed one per nibble.
__device__ __forceinline__ uint32_t e2m1_twice(uint32_t mag3) { return (0xC8643210u >> (mag3 * 4u)) & 15u; }

}  // namespace amx
