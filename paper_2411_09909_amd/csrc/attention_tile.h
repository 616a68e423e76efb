// The per-tile step of the fused quantized attention that both of its kernels share (attention.hip: many queries, K and
// V tiles through LDS; attention_decode.hip: few queries, K and V dequantized in registers): the scores of one tile of
// 32 keys, in the 32x32 accumulator layout of S^T[key, query], become un-normalised probabilities against the running
// row maximum (online softmax), and the 32 probabilities of each query are cast as ONE group (the operands' element and
// scale format) and returned dequantized, as the BF16 B operand of the second product.
//
// Accumulator layout: lane l holds column l % 32 (one query) and rows 8c + 4(l / 32) + r (c, r = 0..3) in register
// 4c + r, so all 32 keys of a query sit in the two lanes l and l ^ 32: the row maximum, the row sum and the group
// maximum of the cast are 16 in-lane steps and one exchange, and registers 8j .. 8j+7, converted to BF16, are the B
// operand of k-step j of P^T's product with V^T staged in that key order.
//
// It is a statement macro, not a function: as an inlined function the same arithmetic compiled to a different
// schedule of the many-queries kernel, 7 % slower (0.735 -> 0.787 ms at 32 / 8 heads x 8192).
#pragma once
#include "cast_math.h"
#include "gemm_common.h"

namespace amx {
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
}  // namespace amx

// Inside a kernel templated on SCALE_KIND. SACC: the tile's raw scores (f32x16); SCALE_LOG2: softmax scale times
// log2(e); MASKED: some key of the tile is masked for some query of the wave (uniform), in which case
// KEY0 + 8 (v / 4) + v % 4 > LIMIT marks register v's key as masked for this lane's query; M, L: the running maximum
// (in units of log2) and sum of this lane's query, updated. Declares PB, the eight words of dequantized probabilities,
// and ALPHA, the factor the query's accumulated output must be multiplied with. EMPTY_OK (a literal): a query may have
// seen no key at all so far; kernels in which every query sees the first key of its first tile pass false.
// P_F16 (a literal; FP8-E5M2 scales only): PB holds FP16 pairs of 2^8 times the dequantized probabilities instead of
// BF16 pairs (exact: at most 6 significant bits, 2^-9 <= 2^8 p <= 2^8, so even the smallest is a normal FP16 number):
// the scale byte is the upper byte of an FP16, so the FP4 -> FP16 conversion and one packed multiply do it.
#define AMX_ATTENTION_TILE_PROBS(EMPTY_OK, SACC, SCALE_LOG2, MASKED, KEY0, LIMIT, M, L, PB, ALPHA, P_F16)          \
    float x[16];                                                                                                   \
    float mx = -__builtin_inff();                                                                                  \
    _Pragma("unroll") for (int v = 0; v < 16; ++v) x[v] = (SACC)[v] * (SCALE_LOG2);                                \
    if (MASKED) { /* uniform over the wave: most tiles skip the masking altogether */                              \
      _Pragma("unroll") for (int v = 0; v < 16; ++v)                                                               \
        if ((KEY0) + 8 * (v >> 2) + (v & 3) > (LIMIT)) x[v] = -__builtin_inff();                                   \
    }                                                                                                              \
    _Pragma("unroll") for (int v = 0; v < 16; ++v) mx = fmaxf(mx, x[v]);                                           \
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                                                                        \
    /* The subtraction below is exact 0 for the score that holds the maximum, so its probability is exactly 1, as  \
       in exact arithmetic (folding the scale into an FMA here would make it 1 - 2^-24 now and then, and a floored \
       power-of-two scale of the tile would halve). */                                                             \
    const float m_raw = fmaxf(M, mx);                                                                              \
    /* EMPTY_OK: a query that has seen no key yet keeps probabilities 0 and alpha 1 instead of the NaN of -inf - -inf */ \
    const float m_new = (EMPTY_OK) && m_raw == -__builtin_inff() ? 0.f : m_raw;                                    \
    const float ALPHA = __builtin_amdgcn_exp2f(M - m_new);                                                         \
    /* exp is monotonic: the largest probability of the tile is the one of the largest score */                    \
    const float pmax = __builtin_amdgcn_exp2f(mx - m_new);                                                         \
    float psum = 0.f;                                                                                              \
    _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                               \
      x[v] = __builtin_amdgcn_exp2f(x[v] - m_new);                                                                 \
      psum += x[v];                                                                                                \
    }                                                                                                              \
    psum += __shfl_xor(psum, 32, 64);                                                                              \
    L = L * ALPHA + psum;                                                                                          \
    M = (EMPTY_OK) ? m_raw : m_new;                                                                                \
    /* cast the 32 probabilities of each query as one group and take the dequantized values as BF16. The quotient  \
       p / S is taken as p * (1 / S): its error of an ulp or two is that of the hardware exp2 which produced p. */ \
    float S, R;                                                                                                    \
    if constexpr (SCALE_KIND == kScaleE5M2 || SCALE_KIND == kScaleE4M3) {                                          \
      fp8_scale_inexact<SCALE_KIND>(pmax, S, R); /* pmax <= 1: no saturation */                                    \
    } else {                                                                                                       \
      (void)encode_scale_sr<SCALE_KIND>(pmax, S, R);                                                               \
    }                                                                                                              \
    uint32_t PB[8];                                                                                                \
    static_assert(!(P_F16) || SCALE_KIND == kScaleE5M2, "FP16 probabilities: FP8-E5M2 scales");                    \
    const _Float16 s_half_ = (_Float16)S; /* exact: an E5M2 value, subnormals included */                          \
    const f16x2 s_half2_ = {s_half_, s_half_};                                                                     \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      if constexpr ((P_F16) && SCALE_KIND == kScaleE5M2) {                                                         \
        const float z0 = x[2 * i] * R, z1 = x[2 * i + 1] * R;                                                      \
        const uint32_t code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(f2u(z0), z0, z1, 1.0f, 0);                  \
        const f16x2 e = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(code, 256.0f, 0);                                 \
        PB[i] = __builtin_bit_cast(uint32_t, e * s_half2_);                                                        \
      } else if constexpr (SCALE_KIND == kScaleE5M2 || SCALE_KIND == kScaleE4M3) {                                 \
        /* the conversion replaces byte 0 of its first operand, the only byte read below: any register will do,    \
           and one that dies here saves the move of a zero */                                                      \
        const float z0 = x[2 * i] * R, z1 = x[2 * i + 1] * R;                                                      \
        const uint32_t code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(f2u(z0), z0, z1, 1.0f, 0);                  \
        const f32x2 e = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 0);                                   \
        /* element * scale has at most 6 significant bits: the truncation to BF16 is exact */                      \
        PB[i] = __builtin_amdgcn_perm(f2u(e[1] * S), f2u(e[0] * S), 0x07060302u);                                  \
      } else {                                                                                                     \
        /* a power-of-two scale is applied by the conversions themselves (they read the exponent field of S: the   \
           first divides by it, the second multiplies) */                                                          \
        const uint32_t code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(f2u(x[2 * i]), x[2 * i], x[2 * i + 1], S, 0); \
        PB[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(code, S, 0));               \
      }                                                                                                            \
    }
