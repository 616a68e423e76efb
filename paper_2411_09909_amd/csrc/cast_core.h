// The cast of BF16 elements held in registers (Appendix B Algorithm 1 with the sign-dependent scale pair of Sec. 4.2
// Eq. 1): shared by the cast kernels and by kernels that cast what they have just computed. A lane holds N / 2 words
// of two BF16 each (N = 8 or 16 consecutive elements of one row); the 2^lanes_log2 neighbouring lanes of a wave hold
// one group. The arithmetic and why it decides as exact arithmetic does: the BF16 section of cast_math.h.
#pragma once
#include "cast_math.h"

namespace amx {

typedef short short2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b) {
  short2v r = __builtin_elementwise_max(__builtin_bit_cast(short2v, a), __builtin_bit_cast(short2v, b));
  return __builtin_bit_cast(uint32_t, r);
}

// max over the 2^lpg_log2 (1, 2, 4 or 8) neighbouring lanes of a group; lpg_log2 is uniform
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v, int lpg_log2) {
  uint32_t o;
  if (lpg_log2 >= 1) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v = v > o ? v : o;
  }
  if (lpg_log2 >= 2) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    v = v > o ? v : o;
  }
  if (lpg_log2 >= 3) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);  // row_half_mirror: lane i <-> 7 - i of 8
    v = v > o ? v : o;
  }
  return v;
}

// the same with two non-negative 16-bit values per register, each half on its own
__device__ __forceinline__ uint32_t group_max_pk16(uint32_t v, int lpg_log2) {
  if (lpg_log2 >= 1) v = pk_max_i16(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true));
  if (lpg_log2 >= 2) v = pk_max_i16(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true));
  if (lpg_log2 >= 3) v = pk_max_i16(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true));
  return v;
}

// Eight BF16 elements (four words, first element in the low half) -> eight E2M1 codes, for an FP8 or power-of-two
// scale given by R ~ 1 / S per sign class (see the BF16 section of cast_math.h): x * R, rounded to binary16, is on the
// same side of every E2M1 boundary as x / S and on it exactly when x / S is; the packed binary16 -> FP4 conversion
// then rounds (nearest, ties to even, sign kept on zero results; it saturates, and a quotient beyond the binary16
// range, which arrives as an infinity, also becomes 6).
template <bool ASYM>
__device__ __forceinline__ uint32_t encode8_bf16(const uint32_t (&d)[4], float r_pos, float r_neg) {
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  uint32_t packed = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float x0 = u2f(d[j] << 16), x1 = u2f(d[j] & 0xFFFF0000u);
    float z0, z1;
    if constexpr (ASYM) {
      z0 = x0 * (x0 < 0.f ? r_neg : r_pos);  // (a negative zero takes r_pos and stays a negative zero)
      z1 = x1 * (x1 < 0.f ? r_neg : r_pos);
    } else {
      z0 = x0 * r_pos;
      z1 = x1 * r_pos;
    }
    const float2v z = {z0, z1};
    const half2v h = __builtin_convertvector(z, half2v);
    if (j == 0) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f16(packed, h, 1.0f, 0);
    if (j == 1) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f16(packed, h, 1.0f, 1);
    if (j == 2) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f16(packed, h, 1.0f, 2);
    if (j == 3) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f16(packed, h, 1.0f, 3);
  }
  return packed;
}

// N BF16 elements of this lane (N / 2 words, first element in the low half of word 0) -> N / 8 words of E2M1 codes
// and the scale byte(s) of the group the lane belongs to (sb_n = sb_p for symmetric formats; every lane of the group
// gets them). Group extrema with packed 16-bit integer maxima: as int16 a negative number's pattern is below zero, so
// max(pattern, 0) keeps the non-negative elements and, after flipping the sign bits, the magnitudes of the negative
// ones. The asymmetric format carries both classes through the lane exchange in one register (positive class in the
// low half, negative in the high half).
template <int SCALE_KIND, bool ASYM, int N>
__device__ __forceinline__ void cast_words_bf16(const uint32_t (&d)[N / 2], int lanes_log2, uint32_t (&code)[N / 8],
                                                uint32_t& sb_p, uint32_t& sb_n) {
  static_assert(N == 8 || N == 16, "8 or 16 elements per lane");
  uint32_t m;
  if constexpr (ASYM) {
    const uint32_t f = 0x80008000u;
    uint32_t p = pk_max_i16(pk_max_i16(d[0], d[1]), pk_max_i16(d[2], d[3]));
    uint32_t n = pk_max_i16(pk_max_i16(d[0] ^ f, d[1] ^ f), pk_max_i16(d[2] ^ f, d[3] ^ f));
    if constexpr (N == 16) {
      p = pk_max_i16(p, pk_max_i16(pk_max_i16(d[4], d[5]), pk_max_i16(d[6], d[7])));
      n = pk_max_i16(n, pk_max_i16(pk_max_i16(d[4] ^ f, d[5] ^ f), pk_max_i16(d[6] ^ f, d[7] ^ f)));
    }
    const uint32_t pl = pk_max_i16(p, p >> 16), nh = pk_max_i16(n, n << 16);
    m = pk_max_i16((pl & 0xFFFFu) | (nh & 0xFFFF0000u), 0u);
  } else {
    const uint32_t k = 0x7FFF7FFFu;
    uint32_t a = pk_max_i16(pk_max_i16(d[0] & k, d[1] & k), pk_max_i16(d[2] & k, d[3] & k));
    if constexpr (N == 16)
      a = pk_max_i16(a, pk_max_i16(pk_max_i16(d[4] & k, d[5] & k), pk_max_i16(d[6] & k, d[7] & k)));
    m = pk_max_i16(a, a >> 16) & 0xFFFFu;
  }
  m = group_max_pk16(m, lanes_log2);
  float r_pos, r_neg;
  sb_p = encode_scale_r_bf16<SCALE_KIND>(u2f(m << 16), r_pos);
  sb_n = sb_p, r_neg = r_pos;
  if constexpr (ASYM) sb_n = encode_scale_r_bf16<SCALE_KIND>(u2f(m & 0xFFFF0000u), r_neg);
#pragma unroll
  for (int t = 0; t < N / 8; ++t) {
    const uint32_t w[4] = {d[4 * t], d[4 * t + 1], d[4 * t + 2], d[4 * t + 3]};
    code[t] = encode8_bf16<ASYM>(w, r_pos, r_neg);
  }
}

}  // namespace amx
