// FP4 codes -> exact 16-bit floats in registers: the dequantization step of the kernels that read an operand as packed
// codes straight from memory (gemm_skinny.hip: the weights of a product with few rows; attention_decode.hip: the keys
// and values of an attention with few queries). element * scale has at most 6 significant bits, so BF16 (and, with a
// bias of 2^-3, FP16 for FP8-E5M2 scales) holds it exactly.
#pragma once
#include "device_formats.h"

namespace amx {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

// all ones in each 16-bit half whose sign bit is set
__device__ __forceinline__ uint32_t pk_sign_mask(uint32_t v) {
  uint32_t m = __builtin_bit_cast(uint32_t, __builtin_bit_cast(i16x2, v) >> (i16x2){15, 15});
  // (an empty statement the optimiser cannot look through: otherwise the mask select that follows is rewritten into
  // two compares, two conditional moves and a byte permute)
  asm("" : "+v"(m));
  return m;
}

// Eight FP4 codes (one word, first code in the lowest nibble) -> eight dequantized 16-bit floats, two per register.
// The scale pair (s_pos, s_neg) comes as bit patterns whose meaning depends on the format (skinny_scales()).
//
// FP8-E5M2 scales, FP16 result biased by 2^-3: the pair holds each scale twice, as packed FP16.
template <bool ASYM, int SEL>
__device__ __forceinline__ uint32_t dequant2_f16(uint32_t word, uint32_t s_pos, uint32_t s_neg) {
  const f16x2 e = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 0.125f, SEL);
  uint32_t sc = s_pos;
  if constexpr (ASYM) {
    const uint32_t m = pk_sign_mask(__builtin_bit_cast(uint32_t, e));
    sc = (s_neg & m) | (s_pos & ~m);
  }
  return __builtin_bit_cast(uint32_t, e * __builtin_bit_cast(f16x2, sc));
}

// Power-of-two scales, BF16 result: the pair holds floats whose exponent field is the scale byte (the conversion
// reads only that field).
template <bool ASYM, int SEL>
__device__ __forceinline__ uint32_t dequant2_pot(uint32_t word, uint32_t s_pos, uint32_t s_neg) {
  const uint32_t p = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, u2f(s_pos), SEL));
  if constexpr (ASYM) {
    const uint32_t n = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, u2f(s_neg), SEL));
    const uint32_t m = pk_sign_mask(p);
    return (n & m) | (p & ~m);
  } else {
    return p;
  }
}

// Any other scale (FP8-E4M3), BF16 result: the pair holds the scales as floats; the hardware FP4 -> FP32 conversion
// gives the signed elements, each is multiplied by the scale of its sign class and the product, which has at most 6
// significant bits, is truncated to BF16 exactly.
template <bool ASYM, int SEL>
__device__ __forceinline__ uint32_t dequant2_f32(uint32_t word, uint32_t s_pos, uint32_t s_neg) {
  const f32x2 e = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, SEL);
  float v0, v1;
  if constexpr (ASYM) {
    const uint32_t m0 = (uint32_t)((int32_t)f2u(e[0]) >> 31), m1 = (uint32_t)((int32_t)f2u(e[1]) >> 31);
    v0 = e[0] * u2f((s_neg & m0) | (s_pos & ~m0));
    v1 = e[1] * u2f((s_neg & m1) | (s_pos & ~m1));
  } else {
    v0 = e[0] * u2f(s_pos);
    v1 = e[1] * u2f(s_pos);
  }
  return __builtin_amdgcn_perm(f2u(v1), f2u(v0), 0x07060302u);  // upper halves: (v0 low, v1 high)
}

template <int SCALE_KIND, bool ASYM>
__device__ __forceinline__ u32x4 dequant_word(uint32_t word, uint32_t s_pos, uint32_t s_neg) {
  if constexpr (SCALE_KIND == kScaleE5M2)
    return u32x4{dequant2_f16<ASYM, 0>(word, s_pos, s_neg), dequant2_f16<ASYM, 1>(word, s_pos, s_neg),
                 dequant2_f16<ASYM, 2>(word, s_pos, s_neg), dequant2_f16<ASYM, 3>(word, s_pos, s_neg)};
  else if constexpr (SCALE_KIND == kScaleE8M0Floor)
    return u32x4{dequant2_pot<ASYM, 0>(word, s_pos, s_neg), dequant2_pot<ASYM, 1>(word, s_pos, s_neg),
                 dequant2_pot<ASYM, 2>(word, s_pos, s_neg), dequant2_pot<ASYM, 3>(word, s_pos, s_neg)};
  else
    return u32x4{dequant2_f32<ASYM, 0>(word, s_pos, s_neg), dequant2_f32<ASYM, 1>(word, s_pos, s_neg),
                 dequant2_f32<ASYM, 2>(word, s_pos, s_neg), dequant2_f32<ASYM, 3>(word, s_pos, s_neg)};
}

}  // namespace amx
