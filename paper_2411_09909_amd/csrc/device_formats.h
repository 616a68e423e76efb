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
    // half -> float by hand: exact for all 3-significant-bit values
    const uint32_t e = (byte >> 2) & 31u, m = byte & 3u;
    if (e == 0) return (float)m * 1.52587890625e-05f;  // m * 2^-16
    return u2f(((e + 112u) << 23) | (m << 21));
  } else if constexpr (SCALE_KIND == kScaleE4M3) {
    const uint32_t e = (byte >> 3) & 15u, m = byte & 7u;
    if (e == 0) return (float)m * 0.001953125f;  // m * 2^-9
    return u2f(((e + 120u) << 23) | (m << 20));
  } else {
    return byte == 0 ? u2f(0x00400000u) : u2f(byte << 23);  // 2^(byte-127)
  }
}

// 2 * |E2M1 value| for the 3-bit magnitude code: {0,1,2,3,4,6,8,12}, packed one per nibble.
__device__ __forceinline__ uint32_t e2m1_twice(uint32_t mag3) { return (0xC8643210u >> (mag3 * 4u)) & 15u; }

}  // namespace amx
