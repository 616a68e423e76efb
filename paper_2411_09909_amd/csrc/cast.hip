// Direct-cast quantization BF16 -> AMXFP4 / MXFP4 (Appendix B Algorithm 1, generalised by Sec. 4.2 Eq. 1 to a
// sign-dependent pair of shared scales) and the matching dequantization (Eq. 1). Group sizes 16, 32, 64, 128 along K
// (Sec. 5.3 / Table 5 compare them; 32 is the paper's choice); scale formats FP8 E5M2 (the paper's), FP8 E4M3 and
// E8M0 with the exponent floored or rounded.
//
// Contiguous cast: one lane owns 8 consecutive BF16 (one 128-bit load); the GS / 8 lanes next to each other own one
// group. Group extrema are found with packed 16-bit integer max (non-negative BF16 patterns order like integers) and
// DPP permutes inside the group. Every decision comes out as exact arithmetic would give it:
//   - an FP8 scale is the correctly rounded FP32 quotient amax/6 rounded once more to 3 (E5M2) or 4 (E4M3)
//     significant bits; the quotient of an 8-bit significand by 3 is either exact or far (>= 2^-13 relative) from
//     every midpoint of that grid, so the two-step rounding equals rounding the real quotient;
//   - the element quotient x / S is formed to within an ulp (exactly when representable, see quotient()) and rounded
//     to E2M1 by the hardware conversion v_cvt_scalef32_pk_fp4_f32.
// Strided cast (groups down a column, for V in P.V): one lane per (row, group), the same arithmetic.
#include "device_formats.h"

namespace amx {

typedef short short2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b) {
  short2v r = __builtin_elementwise_max(__builtin_bit_cast(short2v, a), __builtin_bit_cast(short2v, b));
  return __builtin_bit_cast(uint32_t, r);
}

// max over the 2^lpg_log2 (2, 4, 8 or 16) neighbouring lanes of a group; lpg_log2 is uniform
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v, int lpg_log2) {
  uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
  v = v > o ? v : o;
  if (lpg_log2 >= 2) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    v = v > o ? v : o;
  }
  if (lpg_log2 >= 3) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);  // row_half_mirror: lane i <-> 7 - i of 8
    v = v > o ? v : o;
  }
  if (lpg_log2 >= 4) {
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);  // row_mirror: lane i <-> 15 - i of 16
    v = v > o ? v : o;
  }
  return v;
}

// Shared scale of one sign class: its byte, and the pair (S, R) the element step divides with: S = the scale as a float (exact), R ~ 1/S (0 if S is 0). Power-of-two scales need only R, which is exact.
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_scale_sr(uint32_t amax_bits, float& S, float& R) {
  if constexpr (SCALE_KIND == kScaleE5M2) {
    const float amax = u2f(amax_bits << 16);
    const float q = __fdiv_rn(amax, 6.0f);  // 6 = largest E2M1 magnitude
    int e = (int)(f2u(q) >> 23) - 127;
    e = e < -14 ? -14 : e;  // E5M2 subnormals share the spacing of the lowest normal binade
    // adding 1.5 * 2^(e+21) rounds q to a multiple of 2^(e-2) (nearest, ties to even) in the FP32 adder
    const float magic = u2f(((uint32_t)(e + 21 + 127) << 23) | 0x00400000u);
    float r = (q + magic) - magic;
    r = fminf(r, 57344.0f);
    const uint32_t rb = f2u(r);
    // normal: exponent and two mantissa bits of the float; below 2^-14: m * 2^-16 with m = 0..3
    const uint32_t byte =
        r >= 6.103515625e-05f ? ((((rb >> 23) - 112u) << 2) | ((rb >> 21) & 3u)) : (uint32_t)(r * 65536.0f);
    S = r;
    R = r > 0.f ? __builtin_amdgcn_rcpf(r) : 0.f;
    return byte;
  } else if constexpr (SCALE_KIND == kScaleE4M3) {
    const float amax = u2f(amax_bits << 16);
    const float q = __fdiv_rn(amax, 6.0f);
    int e = (int)(f2u(q) >> 23) - 127;
    e = e < -6 ? -6 : e;  // E4M3 subnormals share the spacing of the lowest normal binade (2^-6)
    // adding 1.5 * 2^(e+20) rounds q to a multiple of 2^(e-3) (nearest, ties to even) in the FP32 adder
    const float magic = u2f(((uint32_t)(e + 20 + 127) << 23) | 0x00400000u);
    float r = (q + magic) - magic;
    r = fminf(r, 448.0f);  // largest finite E4M3 value (byte 0x7E)
    const uint32_t rb = f2u(r);
    // normal: exponent (bias 7) and three mantissa bits of the float; below 2^-6: m * 2^-9 with m = 0..7
    const uint32_t byte = r >= 0.015625f ? ((((rb >> 23) - 120u) << 3) | ((rb >> 20) & 7u)) : (uint32_t)(r * 512.0f);
    S = r;
    R = r > 0.f ? __builtin_amdgcn_rcpf(r) : 0.f;
    return byte;
  } else {
    const uint32_t e8 = amax_bits >> 7, m7 = amax_bits & 127u;
    int b = (int)e8 - 2;
    if constexpr (SCALE_KIND == kScaleE8M0Round) b += (m7 >= 54u) ? 1 : 0;  // significand above sqrt(2)
    b = b < 0 ? 0 : b;
    if (amax_bits == 0) b = 0;
    S = 0.f;                                // unused
    R = u2f((uint32_t)(254 - b) << 23);     // 2^(127 - b) = 1 / scale
    return (uint32_t)b;
  }
}

// x / S for the element step, as a float that rounds to the same E2M1 code as the real quotient:
//  - power-of-two scale: x * R is exact;
//  - FP8 scale: one Newton step on z0 = x * R with the exact residual x - z0 * S (an FMA) gives the quotient to well
//    within an ulp, and exactly when it is representable. Rounding boundaries of E2M1 are representable, and a
//    quotient of an 8-bit by a 3- or 4-bit significand that is not on a boundary is at least 2^-12 (relative) away,
//    so the conversion below decides as exact arithmetic would. S = 0: R = 0 and the result is a zero with x's sign.
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

// Eight elements (four registers of two BF16 each, lower index in the low half) -> eight E2M1 codes, first element
// in the lowest nibble. The E2M1 rounding itself (nearest, ties to even, saturating, sign kept on zero results) is
// done by the packed FP32 -> FP4 conversion instruction.
template <int SCALE_KIND, bool ASYM>
__device__ __forceinline__ uint32_t encode8(const uint32_t (&d)[4], float s_pos, float r_pos, float s_neg,
                                            float r_neg) {
  uint32_t packed = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float x0 = u2f(d[j] << 16), x1 = u2f(d[j] & 0xFFFF0000u);
    float z0, z1;
    if constexpr (ASYM) {
      const bool n0 = (d[j] & 0x8000u) != 0, n1 = (int32_t)d[j] < 0;
      z0 = quotient<SCALE_KIND>(x0, n0 ? s_neg : s_pos, n0 ? r_neg : r_pos);
      z1 = quotient<SCALE_KIND>(x1, n1 ? s_neg : s_pos, n1 ? r_neg : r_pos);
    } else {
      z0 = quotient<SCALE_KIND>(x0, s_pos, r_pos);
      z1 = quotient<SCALE_KIND>(x1, s_pos, r_pos);
    }
    // (the destination byte is an immediate of the instruction)
    if (j == 0) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 0);
    if (j == 1) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 1);
    if (j == 2) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 2);
    if (j == 3) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 3);
  }
  return packed;
}

// Contiguous cast. Thread block = 256 lanes arranged as (256 >> bx_log2) rows x (1 << bx_log2) chunks of 8 elements;
// blockIdx.x walks the rows, blockIdx.y the chunks of a row. A group is 2^lpg_log2 neighbouring lanes; bx is a
// multiple of that and so is the number of chunks in a row, hence a group is always whole and aligned in its wave.
template <int SCALE_KIND, bool ASYM>
__global__ __launch_bounds__(256) void quantize_contig_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                              int64_t row_stride, uint8_t* __restrict__ codes,
                                                              uint8_t* __restrict__ scales, int bx_log2,
                                                              int lpg_log2) {
  const int tx = threadIdx.x & ((1 << bx_log2) - 1), ty = threadIdx.x >> bx_log2;
  const int64_t r = (int64_t)blockIdx.x * (256 >> bx_log2) + ty;
  const int cc = (int)(blockIdx.y << bx_log2) + tx;  // chunk of 8 elements within the row
  if (r >= rows || cc >= (int)(K >> 3)) return;
  const uint4 v = *reinterpret_cast<const uint4*>(x + r * row_stride + (int64_t)cc * 8);
  const uint32_t d[4] = {v.x, v.y, v.z, v.w};
  // group extrema (steps "max_i |V_i|" of Algorithm 1, split by sign for the asymmetric format)
  uint32_t amax_p, amax_n;
  if constexpr (ASYM) {
    uint32_t p = pk_max_i16(pk_max_i16(d[0], d[1]), pk_max_i16(d[2], d[3]));
    p = pk_max_i16(p, 0u);  // negative patterns (sign bit set) compare below zero as int16
    uint32_t n = pk_max_i16(pk_max_i16(d[0] ^ 0x80008000u, d[1] ^ 0x80008000u),
                            pk_max_i16(d[2] ^ 0x80008000u, d[3] ^ 0x80008000u));
    n = pk_max_i16(n, 0u);
    amax_p = (p & 0xFFFFu) > (p >> 16) ? (p & 0xFFFFu) : (p >> 16);
    amax_n = (n & 0xFFFFu) > (n >> 16) ? (n & 0xFFFFu) : (n >> 16);
    amax_p = group_max_u32(amax_p, lpg_log2);
    amax_n = group_max_u32(amax_n, lpg_log2);
  } else {
    uint32_t a = pk_max_i16(pk_max_i16(d[0] & 0x7FFF7FFFu, d[1] & 0x7FFF7FFFu),
                            pk_max_i16(d[2] & 0x7FFF7FFFu, d[3] & 0x7FFF7FFFu));
    amax_p = (a & 0xFFFFu) > (a >> 16) ? (a & 0xFFFFu) : (a >> 16);
    amax_p = group_max_u32(amax_p, lpg_log2);
    amax_n = amax_p;
  }
  float s_pos, r_pos, s_neg, r_neg;
  const uint32_t sb_p = encode_scale_sr<SCALE_KIND>(amax_p, s_pos, r_pos);
  uint32_t sb_n = sb_p;
  s_neg = s_pos, r_neg = r_pos;
  if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(amax_n, s_neg, r_neg);
  *reinterpret_cast<uint32_t*>(codes + r * (K >> 1) + (int64_t)cc * 4) =
      encode8<SCALE_KIND, ASYM>(d, s_pos, r_pos, s_neg, r_neg);
  if ((tx & ((1 << lpg_log2) - 1)) == 0) {
    const int64_t g = r * (K >> (lpg_log2 + 3)) + (cc >> lpg_log2);
    if constexpr (ASYM)
      *reinterpret_cast<uint16_t*>(scales + g * 2) = (uint16_t)(sb_p | (sb_n << 8));
    else
      scales[g] = (uint8_t)sb_p;
  }
}

// Groups run down a column: element (r, k) = x[r + k * k_stride]. One lane owns one (row, group) of GS elements;
// consecutive lanes own consecutive rows, so each of the GS loads of a wave reads 128 contiguous bytes.
template <int SCALE_KIND, bool ASYM, int GS>
__global__ __launch_bounds__(256) void quantize_strided_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                               int64_t k_stride, uint8_t* __restrict__ codes,
                                                               uint8_t* __restrict__ scales) {
  const int64_t G = K / GS;
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t g = blockIdx.y;
  if (r >= rows) return;
  const uint16_t* p = x + r + g * GS * k_stride;
  uint32_t d[GS / 2];  // two elements per register, lower index in the low half
  uint32_t amax_p = 0, amax_n = 0;
#pragma unroll
  for (int i = 0; i < GS; i += 2) {
    const uint32_t b0 = p[i * k_stride], b1 = p[(i + 1) * k_stride];
    d[i >> 1] = b0 | (b1 << 16);
    const uint32_t m0 = b0 & 0x7FFFu, m1 = b1 & 0x7FFFu;
    if (b0 & 0x8000u)
      amax_n = m0 > amax_n ? m0 : amax_n;
    else
      amax_p = m0 > amax_p ? m0 : amax_p;
    if (b1 & 0x8000u)
      amax_n = m1 > amax_n ? m1 : amax_n;
    else
      amax_p = m1 > amax_p ? m1 : amax_p;
  }
  if constexpr (!ASYM) amax_p = amax_n = (amax_p > amax_n ? amax_p : amax_n);
  float s_pos, r_pos, s_neg, r_neg;
  const uint32_t sb_p = encode_scale_sr<SCALE_KIND>(amax_p, s_pos, r_pos);
  uint32_t sb_n = sb_p;
  s_neg = s_pos, r_neg = r_pos;
  if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(amax_n, s_neg, r_neg);
  uint32_t* out = reinterpret_cast<uint32_t*>(codes + r * (K >> 1) + g * (GS / 2));
#pragma unroll
  for (int t = 0; t < GS / 16; ++t) {
    const uint32_t lo[4] = {d[8 * t], d[8 * t + 1], d[8 * t + 2], d[8 * t + 3]};
    const uint32_t hi[4] = {d[8 * t + 4], d[8 * t + 5], d[8 * t + 6], d[8 * t + 7]};
    *reinterpret_cast<uint2*>(out + 2 * t) = make_uint2(encode8<SCALE_KIND, ASYM>(lo, s_pos, r_pos, s_neg, r_neg),
                                                        encode8<SCALE_KIND, ASYM>(hi, s_pos, r_pos, s_neg, r_neg));
  }
  if constexpr (ASYM)
    *reinterpret_cast<uint16_t*>(scales + (r * G + g) * 2) = (uint16_t)(sb_p | (sb_n << 8));
  else
    scales[r * G + g] = (uint8_t)sb_p;
}

// x_hat = (-1)^s * elem * S_class (Eq. 1). One lane expands 8 codes.
template <int SCALE_KIND, bool ASYM, bool OUT_BF16>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t* __restrict__ codes,
                                                         const uint8_t* __restrict__ scales, int64_t rows, int64_t K,
                                                         int gs_log2, void* __restrict__ out) {
  const int64_t chunks_per_row = K >> 3;
  const int64_t total = rows * chunks_per_row;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < total; c += (int64_t)gridDim.x * 256) {
    const int64_t r = c / chunks_per_row;
    const int64_t cc = c - r * chunks_per_row;
    const uint32_t w = *reinterpret_cast<const uint32_t*>(codes + r * (K >> 1) + cc * 4);
    const int64_t g = r * (K >> gs_log2) + ((cc * 8) >> gs_log2);
    float s_pos, s_neg;
    if constexpr (ASYM) {
      const uint32_t sb = *reinterpret_cast<const uint16_t*>(scales + g * 2);
      s_pos = scale_value<SCALE_KIND>(sb & 255u);
      s_neg = scale_value<SCALE_KIND>(sb >> 8);
    } else {
      s_pos = s_neg = scale_value<SCALE_KIND>(scales[g]);
    }
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t n = (w >> (4 * j)) & 15u;
      const float mag2 = (float)e2m1_twice(n & 7u);  // 2 * |element|
      const float s = (n & 8u) ? -0.5f * s_neg : 0.5f * s_pos;
      v[j] = mag2 * s;  // <= 5 significant bits: exact in FP32 and in BF16
    }
    if constexpr (OUT_BF16) {
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = (f2u(v[2 * j]) >> 16) | (f2u(v[2 * j + 1]) & 0xFFFF0000u);
      *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(out) + r * K + cc * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      float4* o = reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + r * K + cc * 8);
      o[0] = make_float4(v[0], v[1], v[2], v[3]);
      o[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
  }
}

static int grid_for(int64_t total_threads) {
  int64_t blocks = (total_threads + 255) / 256;
  const int64_t cap = 256 * 32;  // 256 CUs x 32 resident blocks of 256: grid-stride beyond that
  return (int)(blocks < cap ? blocks : cap);
}

// log2 of a supported group size (16, 32, 64, 128), else -1
static int group_log2(int64_t gs) { return gs == 16 ? 4 : gs == 32 ? 5 : gs == 64 ? 6 : gs == 128 ? 7 : -1; }

template <int SK, bool ASYM>
static hipError_t launch_qc(const uint16_t* x, int64_t rows, int64_t K, int gs_log2, int64_t row_stride,
                            uint8_t* codes, uint8_t* scales, hipStream_t s) {
  // block shape: as many chunks of a row as fit (power of two, one group .. 256), the rest of the 256 lanes go to
  // more rows
  const int64_t chunks = K / 8;
  const int lpg_log2 = gs_log2 - 3;
  int bx_log2 = lpg_log2 < 2 ? 2 : lpg_log2;
  while (bx_log2 < 8 && (int64_t(1) << (bx_log2 + 1)) <= chunks) ++bx_log2;
  const int64_t bx = int64_t(1) << bx_log2, by = 256 >> bx_log2;
  hipLaunchKernelGGL((quantize_contig_kernel<SK, ASYM>), dim3((unsigned)((rows + by - 1) / by),
                     (unsigned)((chunks + bx - 1) / bx)), dim3(256), 0, s, x, rows, K, row_stride, codes, scales,
                     bx_log2, lpg_log2);
  return hipGetLastError();
}

// Calls f.template operator()<SCALE_KIND, ASYM>() for the run-time pair (scale_kind, asym).
template <class F>
static hipError_t for_format(int scale_kind, bool asym, F&& f) {
  switch (scale_kind) {
    case kScaleE5M2:
      return asym ? f.template operator()<kScaleE5M2, true>() : f.template operator()<kScaleE5M2, false>();
    case kScaleE4M3:
      return asym ? f.template operator()<kScaleE4M3, true>() : f.template operator()<kScaleE4M3, false>();
    case kScaleE8M0Floor:
      return asym ? f.template operator()<kScaleE8M0Floor, true>() : f.template operator()<kScaleE8M0Floor, false>();
    case kScaleE8M0Round:
      return asym ? f.template operator()<kScaleE8M0Round, true>() : f.template operator()<kScaleE8M0Round, false>();
  }
  return hipErrorInvalidValue;
}

hipError_t launch_quantize_contig(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, int64_t rows,
                                  int64_t K, int64_t row_stride, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || K % group_size != 0) return hipErrorInvalidValue;
  return for_format(scale_kind, asym, [&]<int SK, bool ASYM>() {
    return launch_qc<SK, ASYM>(x, rows, K, gl, row_stride, codes, scales, s);
  });
}

template <int SK, bool ASYM, int GS>
static hipError_t launch_qs(const uint16_t* x, int64_t rows, int64_t K, int64_t k_stride, uint8_t* codes,
                            uint8_t* scales, hipStream_t s) {
  hipLaunchKernelGGL((quantize_strided_kernel<SK, ASYM, GS>), dim3((unsigned)((rows + 255) / 256), (unsigned)(K / GS)),
                     dim3(256), 0, s, x, rows, K, k_stride, codes, scales);
  return hipGetLastError();
}

hipError_t launch_quantize_strided(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, int64_t rows,
                                   int64_t K, int64_t k_stride, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || K % group_size != 0) return hipErrorInvalidValue;
  return for_format(scale_kind, asym, [&]<int SK, bool ASYM>() {
    switch (gl) {
      case 4: return launch_qs<SK, ASYM, 16>(x, rows, K, k_stride, codes, scales, s);
      case 5: return launch_qs<SK, ASYM, 32>(x, rows, K, k_stride, codes, scales, s);
      case 6: return launch_qs<SK, ASYM, 64>(x, rows, K, k_stride, codes, scales, s);
      default: return launch_qs<SK, ASYM, 128>(x, rows, K, k_stride, codes, scales, s);
    }
  });
}

template <int SK, bool ASYM>
static hipError_t launch_dq(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K, int gs_log2,
                            void* out, int out_dtype, hipStream_t s) {
  const dim3 grid(grid_for(rows * (K / 8)));
  if (out_dtype == 1)
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, true>), grid, dim3(256), 0, s, codes, scales, rows, K, gs_log2,
                       out);
  else
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, false>), grid, dim3(256), 0, s, codes, scales, rows, K, gs_log2,
                       out);
  return hipGetLastError();
}

hipError_t launch_dequantize(int scale_kind, bool asym, int64_t group_size, const uint8_t* codes,
                             const uint8_t* scales, int64_t rows, int64_t K, void* out, int out_dtype, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || K % group_size != 0) return hipErrorInvalidValue;
  // E8M0 floor and round share the byte encoding
  return for_format(scale_kind == kScaleE8M0Round ? kScaleE8M0Floor : scale_kind, asym, [&]<int SK, bool ASYM>() {
    return launch_dq<SK, ASYM>(codes, scales, rows, K, gl, out, out_dtype, s);
  });
}

}  // namespace amx
