// Arithmetic of the direct cast on register values (Appendix B Algorithm 1 with the scale formats of Sec. 4.2): the
// shared scale of a group from its largest magnitude, and the element quotient that the FP4 conversion instruction
// then rounds. Used by the cast kernels and by kernels that cast values they have just computed.
#pragma once
#include "device_formats.h"

namespace amx {

// FP8 shared scale (MBITS mantissa bits, smallest normal exponent EMIN, exponent bias BIAS, largest value maxv) of a
// sign class with largest magnitude amax >= 0 (any FP32 number): the real quotient amax / 6 (6 = largest E2M1
// magnitude) rounded to nearest, ties to even, saturating, subnormals kept. q is the correctly rounded FP32 quotient;
// adding 1.5 * 2^(e+23-MBITS) rounds it to a multiple of 2^(e-MBITS) in the FP32 adder. The two-step rounding equals
// rounding the real quotient: neighbouring FP32 values of amax are 4 or 8 ulps of q apart, so their quotients differ
// by 2/3 or 4/3 ulp of q, and q lands on a midpoint of the FP8 grid only when amax / 6 is that midpoint exactly.
template <int MBITS, int EMIN, int BIAS>
__device__ __forceinline__ uint32_t fp8_scale(float amax, float maxv, float& S, float& R) {
  const float q = __fdiv_rn(amax, 6.0f);
  int e = (int)(f2u(q) >> 23) - 127;
  e = e < EMIN ? EMIN : e;  // subnormals share the spacing of the lowest normal binade
  const float magic = u2f(((uint32_t)(e + 23 - MBITS + 127) << 23) | 0x00400000u);
  float r = (q + magic) - magic;
  r = fminf(r, maxv);
  const uint32_t rb = f2u(r);
  // normal: exponent and MBITS mantissa bits of the float; below 2^EMIN: m * 2^(EMIN - MBITS)
  const float min_normal = u2f((uint32_t)(EMIN + 127) << 23), to_int = u2f((uint32_t)(MBITS - EMIN + 127) << 23);
  const uint32_t byte = r >= min_normal
                            ? ((((rb >> 23) - (uint32_t)(127 - BIAS)) << MBITS) | ((rb >> (23 - MBITS)) & ((1u << MBITS) - 1u)))
                            : (uint32_t)(r * to_int);
  S = r;
  R = r > 0.f ? __builtin_amdgcn_rcpf(r) : 0.f;
  return byte;
}

// Shared scale of one sign class with largest magnitude amax (a non-negative float): its byte, and the pair (S, R)
// the element step divides with: S = the scale as a float (exact), R ~ 1/S (0 if S is 0; exact for power-of-two
// scales, which divide by multiplying with R alone).
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_scale_sr(float amax, float& S, float& R) {
  if constexpr (SCALE_KIND == kScaleE5M2) {
    return fp8_scale<2, -14, 15>(amax, 57344.0f, S, R);
  } else if constexpr (SCALE_KIND == kScaleE4M3) {
    return fp8_scale<3, -6, 7>(amax, 448.0f, S, R);  // 448 = largest finite E4M3 value (byte 0x7E)
  } else {
    const uint32_t bits = f2u(amax), e8 = bits >> 23, m23 = bits & 0x7FFFFFu;
    int b = (int)e8 - 2;
    // exponent rounded instead of floored: one more when the significand exceeds sqrt(2) = 1 + 3474675.3 / 2^23
    if constexpr (SCALE_KIND == kScaleE8M0Round) b += (m23 >= 3474676u) ? 1 : 0;
    b = b < 0 ? 0 : b;
    if (bits == 0) b = 0;
    S = b == 0 ? u2f(0x00400000u) : u2f((uint32_t)b << 23);  // 2^(b - 127); byte 0 is an FP32 subnormal
    R = u2f((uint32_t)(254 - b) << 23);                       // 2^(127 - b) = 1 / scale
    return (uint32_t)b;
  }
}

// x / S for the element step (x any FP32 number), as a float that rounds to the same E2M1 code as the real quotient:
//  - power-of-two scale: x * R is exact;
//  - FP8 scale: one Newton step on z0 = x * R with the exact residual x - z0 * S (an FMA) gives the correctly rounded
//    quotient except within 2^-20 ulp of a rounding midpoint of FP32, and the exact one when it is representable.
//    The E2M1 rounding boundaries b are representable. If x / S is not b, x differs from b * S (at most 7
//    significant bits) by at least an ulp of x, which is between 0.53 and 2 ulps of the quotient for the significands
//    an FP8 scale can have (1/1.875 at worst): the quotient is at least 0.53 ulp from b, never rounds onto it, and the
//    conversion below decides as exact arithmetic would. S = 0: R = 0 and the result is a zero with x's sign.
template <int SCALE_KIND>
__device__ __forceinline__ float quotient(float x, float S, float R) {
  const float z0 = x * R;
  if constexpr (SCALE_KIND == kScaleE5M2 || SCALE_KIND == kScaleE4M3) {
    const float res = __builtin_fmaf(-z0, S, x);
    // (x = -0 gives res = +0 and the sum below would lose the sign, which the code keeps: put it back)
    return __builtin_copysignf(__builtin_fmaf(res, R, z0), x);
  } else {
    return z0;
  }
}

// ---- BF16 inputs -----------------------------------------------------------------------------------------------
// When the elements are BF16 numbers (8 significant bits) the exact decisions need less arithmetic, because a
// quantity that is not exactly on a rounding boundary is far from it:
//  - scale: a boundary t of the FP8 grid has MBITS + 2 significant bits, so 6 t is a multiple of the BF16 spacing
//    around it and amax != 6 t implies |amax / 6 - t| >= 2^-8.5 t. The product amax * fl(1/6) (relative error below
//    2^-22), snapped to 13 significant bits, therefore lies on the same side of every boundary as amax / 6, and
//    lands on the boundary exactly when amax / 6 does; the hardware FP8 conversion (nearest, ties to even,
//    subnormals kept) then rounds as the real quotient would be rounded.
//  - element: an E2M1 boundary b times the scale has at most 7 significant bits, so x != b S implies
//    |x / S - b| >= 2^-9 b. The product x * R with R = rcp(S) (relative error below 2^-21), rounded to binary16
//    (11 significant bits), keeps its side of every boundary and is b exactly when x / S is; see encode8_bf16()
//    in cast_core.h.

typedef float float2v __attribute__((ext_vector_type(2)));

// FP8 scale byte (MBITS = 2: E5M2, 3: E4M3) of a sign class whose largest magnitude amax is a BF16 number, and
// R ~ 1 / scale (0 when the scale is 0).
template <int MBITS>
__device__ __forceinline__ uint32_t fp8_scale_bf16(float amax, float& R) {
  const float q0 = amax * 0x1.555556p-3f;                               // ~ amax / 6
  uint32_t qb = (f2u(q0) + 0x400u) & 0xFFFFF800u;                      // 13 significant bits
  const uint32_t maxb = MBITS == 2 ? 0x47600000u : 0x43E00000u;         // 57344, 448: the largest finite scale
  qb = qb < maxb ? qb : maxb;                                           // (non-negative floats order like integers)
  const float q = u2f(qb);
  uint32_t byte;
  float S;
  if constexpr (MBITS == 2) {
    byte = (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(q, q, 0, false) & 0xFFu;
    S = (float)__builtin_bit_cast(_Float16, (uint16_t)(byte << 8));
  } else {
    byte = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(q, q, 0, false) & 0xFFu;
    S = (float)__builtin_bit_cast(_Float16, (uint16_t)(byte << 7)) * 256.0f;
  }
  R = byte ? __builtin_amdgcn_rcpf(S) : 0.f;
  return byte;
}

// encode_scale_sr() for a BF16 amax: byte and R only (the element step needs no S).
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_scale_r_bf16(float amax, float& R) {
  if constexpr (SCALE_KIND == kScaleE5M2) {
    return fp8_scale_bf16<2>(amax, R);
  } else if constexpr (SCALE_KIND == kScaleE4M3) {
    return fp8_scale_bf16<3>(amax, R);
  } else {
    float S;
    return encode_scale_sr<SCALE_KIND>(amax, S, R);
  }
}

// FP8 scale of a magnitude that is itself only accurate to an ulp or two (a probability out of the hardware exp2):
// S = the hardware FP8 conversion (nearest, ties to even, subnormals kept) of amax * fl(1/6), R ~ 1 / S (0 when S is
// 0). amax must be small enough for amax / 6 to be a finite scale (probabilities are at most 1). Against the exact
// quotient the product is off by one more ulp of FP32, which moves the rounded scale only where the inexact amax
// already could.
template <int SCALE_KIND>
__device__ __forceinline__ void fp8_scale_inexact(float amax, float& S, float& R) {
  static_assert(SCALE_KIND == kScaleE5M2 || SCALE_KIND == kScaleE4M3, "FP8 scales only");
  const float q = amax * 0x1.555556p-3f;
  uint32_t byte;
  if constexpr (SCALE_KIND == kScaleE5M2) {
    byte = (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(q, q, 0, false) & 0xFFu;
    S = (float)__builtin_bit_cast(_Float16, (uint16_t)(byte << 8));
  } else {
    byte = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(q, q, 0, false) & 0xFFu;
    S = (float)__builtin_bit_cast(_Float16, (uint16_t)(byte << 7)) * 256.0f;
  }
  R = byte ? __builtin_amdgcn_rcpf(S) : 0.f;
}

}  // namespace amx
