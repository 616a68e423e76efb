// Direct-cast quantization BF16 -> AMXFP4 / MXFP4 (Appendix B Algorithm 1, generalised by Sec. 4.2 Eq. 1 to a
// sign-dependent pair of shared scales) and the matching dequantization (Eq. 1).
//
// Contiguous cast: one lane owns 8 consecutive BF16 (one 128-bit load); the 4 lanes of a quad own one group of 32.
// Group extrema are found with packed 16-bit integer max (non-negative BF16 patterns order like integers) and two
// DPP quad permutes. Every decision comes out as exact arithmetic would give it:
//   - the E5M2 scale is the correctly rounded FP32 quotient amax/6 rounded once more to 3 significant bits; the
//     quotient of an 8-bit significand by 3 is either exact or far (>= 2^-12 relative) from every 4-bit midpoint,
//     so the two-step rounding equals rounding the real quotient;
//   - contiguous kernel: the element quotient x / S is formed to within an ulp (exactly when representable, see
//     quotient()) and rounded to E2M1 by the hardware conversion v_cvt_scalef32_pk_fp4_f32;
//   - strided kernel: an element is compared as y = |x| * (420/M) * 2^-e against the fixed thresholds 420 * {.25,
//     .75,1.25,1.75,2.5,3.5,5}, where the scale is M * 2^e with integer M in 1..7: 420 = lcm(1..7) makes y an exact
//     FP32 product (8-bit x 9-bit significands), so no division and no reciprocal rounding is involved.
#include "device_formats.h"

namespace amx {

typedef short short2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b) {
  short2v r = __builtin_elementwise_max(__builtin_bit_cast(short2v, a), __builtin_bit_cast(short2v, b));
  return __builtin_bit_cast(uint32_t, r);
}

// max over the 4 lanes of a quad
__device__ __forceinline__ uint32_t quad_max_u32(uint32_t v) {
  uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
  v = v > o ? v : o;
  o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);           // quad_perm [2,3,0,1]
  return v > o ? v : o;
}

// Shared-scale byte for a sign class with largest magnitude `amax_bits` (BF16 pattern, sign clear), and the factor
// `kfac` such that y = |x| * kfac is compared against UNIT * t (UNIT = 420 for FP8 scales, 1 for power-of-two scales).
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_scale(uint32_t amax_bits, float& kfac) {
  if constexpr (SCALE_KIND == kScaleE5M2) {
    if (amax_bits == 0) {
      kfac = 0.f;
      return 0;
    }
    const float amax = u2f(amax_bits << 16);
    const float q = __fdiv_rn(amax, 6.0f);  // 6 = largest E2M1 magnitude
    int e = (int)(f2u(q) >> 23) - 127;
    e = e < -14 ? -14 : e;  // E5M2 subnormals share the spacing of the lowest normal binade
    // adding 1.5 * 2^(e+21) rounds q to a multiple of 2^(e-2) (nearest, ties to even) in the FP32 adder
    const float magic = u2f(((uint32_t)(e + 21 + 127) << 23) | 0x00400000u);
    float r = (q + magic) - magic;
    r = fminf(r, 57344.0f);
    const uint32_t rb = f2u(r);
    uint32_t byte;
    if (r >= 6.103515625e-05f) {  // 2^-14: normal
      byte = (((rb >> 23) - 112u) << 2) | ((rb >> 21) & 3u);
      const uint32_t m = byte & 3u, e5 = byte >> 2;
      const uint32_t c = (0x3C465469u >> (8u * m)) & 255u;  // 420 / (4 + m) = 105, 84, 70, 60
      kfac = u2f(f2u((float)c) + ((17u - e5) << 23));       // c * 2^(17 - e5); scale = (4+m) * 2^(e5-17)
    } else {
      byte = (uint32_t)(r * 65536.0f);  // m * 2^-16, m in 0..3
      const float c = byte == 1 ? 420.f : (byte == 2 ? 210.f : 140.f);
      kfac = byte == 0 ? 0.f : c * 65536.0f;
    }
    return byte;
  } else {
    const uint32_t e8 = amax_bits >> 7, m7 = amax_bits & 127u;
    int b = (int)e8 - 2;
    if constexpr (SCALE_KIND == kScaleE8M0Round) b += (m7 >= 54u) ? 1 : 0;  // significand above sqrt(2)
    b = b < 0 ? 0 : b;
    if (amax_bits == 0) b = 0;
    kfac = u2f((uint32_t)(254 - b) << 23);  // 2^(127 - b) = 1 / scale
    return (uint32_t)b;
  }
}

// 3-bit E2M1 magnitude code of y / UNIT (nearest, ties to the even code, saturating at 6).
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_mag(float y) {
  constexpr float U = (SCALE_KIND == kScaleE5M2) ? 420.f : 1.f;
  uint32_t c = 0;
  c += (y > 0.25f * U) ? 1u : 0u;
  c += (y >= 0.75f * U) ? 1u : 0u;
  c += (y > 1.25f * U) ? 1u : 0u;
  c += (y >= 1.75f * U) ? 1u : 0u;
  c += (y > 2.5f * U) ? 1u : 0u;
  c += (y >= 3.5f * U) ? 1u : 0u;
  c += (y > 5.0f * U) ? 1u : 0u;
  return c;
}

// code nibble of one BF16 pattern
template <int SCALE_KIND>
__device__ __forceinline__ uint32_t encode_elem(uint32_t bits16, float k_pos, float k_neg) {
  const uint32_t neg = bits16 >> 15;
  const float ax = u2f((bits16 & 0x7FFFu) << 16);
  const float y = ax * (neg ? k_neg : k_pos);
  return (neg << 3) | encode_mag<SCALE_KIND>(y);
}

// Shared scale of one sign class for the contiguous kernel: its byte, and the pair (S, R) the element step divides
// with: S = the scale as a float (exact), R ~ 1/S (0 if S is 0). Power-of-two scales need only R, which is exact.
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
//    quotient of an 8-bit by a 3-bit significand that is not on a boundary is at least 2^-11 (relative) away from it,
//    so the conversion below decides as exact arithmetic would. S = 0: R = 0 and the result is a zero with x's sign.
template <int SCALE_KIND>
__device__ __forceinline__ float quotient(float x, float S, float R) {
  const float z0 = x * R;
  if constexpr (SCALE_KIND == kScaleE5M2) {
    const float res = __builtin_fmaf(-z0, S, x);
    // (x = -0 gives res = +0 and the sum below would lose the sign, which the code keeps: put it back)
    return __builtin_copysignf(__builtin_fmaf(res, R, z0), x);
  } else {
    return z0;
  }
}

// Contiguous cast. Thread block = 256 lanes arranged as (256 >> bx_log2) rows x (1 << bx_log2) chunks of 8 elements;
// blockIdx.x walks the rows, blockIdx.y the chunks of a row. bx is a multiple of 4 and so is the number of chunks in
// a row, hence a quad (one group) is always whole. The E2M1 rounding itself (nearest, ties to even, saturating, sign
// kept on zero results) is done by the packed FP32 -> FP4 conversion instruction.
template <int SCALE_KIND, bool ASYM>
__global__ __launch_bounds__(256) void quantize_contig_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                              int64_t row_stride, uint8_t* __restrict__ codes,
                                                              uint8_t* __restrict__ scales, int bx_log2) {
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
    amax_p = quad_max_u32(amax_p);
    amax_n = quad_max_u32(amax_n);
  } else {
    uint32_t a = pk_max_i16(pk_max_i16(d[0] & 0x7FFF7FFFu, d[1] & 0x7FFF7FFFu),
                            pk_max_i16(d[2] & 0x7FFF7FFFu, d[3] & 0x7FFF7FFFu));
    amax_p = (a & 0xFFFFu) > (a >> 16) ? (a & 0xFFFFu) : (a >> 16);
    amax_p = quad_max_u32(amax_p);
    amax_n = amax_p;
  }
  float s_pos, r_pos, s_neg, r_neg;
  const uint32_t sb_p = encode_scale_sr<SCALE_KIND>(amax_p, s_pos, r_pos);
  uint32_t sb_n = sb_p;
  s_neg = s_pos, r_neg = r_pos;
  if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(amax_n, s_neg, r_neg);
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
    if (j == 0) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 0);
    if (j == 1) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 1);
    if (j == 2) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 2);
    if (j == 3) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, z0, z1, 1.0f, 3);
  }
  *reinterpret_cast<uint32_t*>(codes + r * (K >> 1) + (int64_t)cc * 4) = packed;
  if ((tx & 3) == 0) {
    const int64_t g = r * (K >> 5) + (cc >> 2);
    if constexpr (ASYM)
      *reinterpret_cast<uint16_t*>(scales + g * 2) = (uint16_t)(sb_p | (sb_n << 8));
    else
      scales[g] = (uint8_t)sb_p;
  }
}

// Groups run down a column: element (r, k) = x[r + k * k_stride]. One lane owns one (row, group); consecutive lanes
// own consecutive rows, so each of the 32 loads of a wave reads 128 contiguous bytes.
template <int SCALE_KIND, bool ASYM>
__global__ __launch_bounds__(256) void quantize_strided_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                               int64_t k_stride, uint8_t* __restrict__ codes,
                                                               uint8_t* __restrict__ scales) {
  const int64_t G = K >> 5;
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t g = blockIdx.y;
  if (r >= rows) return;
  const uint16_t* p = x + r + g * 32 * k_stride;
  uint32_t b[32];
  uint32_t amax_p = 0, amax_n = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    b[i] = p[i * k_stride];
    const uint32_t mag = b[i] & 0x7FFFu;
    if (b[i] & 0x8000u)
      amax_n = mag > amax_n ? mag : amax_n;
    else
      amax_p = mag > amax_p ? mag : amax_p;
  }
  if constexpr (!ASYM) amax_p = amax_n = (amax_p > amax_n ? amax_p : amax_n);
  float k_pos, k_neg;
  const uint32_t sb_p = encode_scale<SCALE_KIND>(amax_p, k_pos);
  uint32_t sb_n = sb_p;
  k_neg = k_pos;
  if constexpr (ASYM) sb_n = encode_scale<SCALE_KIND>(amax_n, k_neg);
  uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 32; ++i) w[i >> 3] |= encode_elem<SCALE_KIND>(b[i], k_pos, k_neg) << (4 * (i & 7));
  *reinterpret_cast<uint4*>(codes + r * (K >> 1) + g * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  if constexpr (ASYM)
    *reinterpret_cast<uint16_t*>(scales + (r * G + g) * 2) = (uint16_t)(sb_p | (sb_n << 8));
  else
    scales[r * G + g] = (uint8_t)sb_p;
}

// x_hat = (-1)^s * elem * S_class (Eq. 1). One lane expands 8 codes.
template <int SCALE_KIND, bool ASYM, bool OUT_BF16>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t* __restrict__ codes,
                                                         const uint8_t* __restrict__ scales, int64_t rows, int64_t K,
                                                         void* __restrict__ out) {
  const int64_t chunks_per_row = K >> 3;
  const int64_t total = rows * chunks_per_row;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < total; c += (int64_t)gridDim.x * 256) {
    const int64_t r = c / chunks_per_row;
    const int64_t cc = c - r * chunks_per_row;
    const uint32_t w = *reinterpret_cast<const uint32_t*>(codes + r * (K >> 1) + cc * 4);
    const int64_t g = r * (K >> 5) + (cc >> 2);
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

template <int SK, bool ASYM>
static hipError_t launch_qc(const uint16_t* x, int64_t rows, int64_t K, int64_t row_stride, uint8_t* codes,
                            uint8_t* scales, hipStream_t s) {
  // block shape: as many chunks of a row as fit (power of two, 4 .. 256), the rest of the 256 lanes go to more rows
  const int64_t chunks = K / 8;
  int bx_log2 = 2;
  while (bx_log2 < 8 && (int64_t(1) << (bx_log2 + 1)) <= chunks) ++bx_log2;
  const int64_t bx = int64_t(1) << bx_log2, by = 256 >> bx_log2;
  hipLaunchKernelGGL((quantize_contig_kernel<SK, ASYM>), dim3((unsigned)((rows + by - 1) / by),
                     (unsigned)((chunks + bx - 1) / bx)), dim3(256), 0, s, x, rows, K, row_stride, codes, scales,
                     bx_log2);
  return hipGetLastError();
}

hipError_t launch_quantize_contig(int scale_kind, bool asym, const uint16_t* x, int64_t rows, int64_t K,
                                  int64_t row_stride, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  switch (scale_kind) {
    case kScaleE5M2:
      return asym ? launch_qc<kScaleE5M2, true>(x, rows, K, row_stride, codes, scales, s)
                  : launch_qc<kScaleE5M2, false>(x, rows, K, row_stride, codes, scales, s);
    case kScaleE8M0Floor:
      return asym ? launch_qc<kScaleE8M0Floor, true>(x, rows, K, row_stride, codes, scales, s)
                  : launch_qc<kScaleE8M0Floor, false>(x, rows, K, row_stride, codes, scales, s);
    case kScaleE8M0Round:
      return asym ? launch_qc<kScaleE8M0Round, true>(x, rows, K, row_stride, codes, scales, s)
                  : launch_qc<kScaleE8M0Round, false>(x, rows, K, row_stride, codes, scales, s);
  }
  return hipErrorInvalidValue;
}

template <int SK, bool ASYM>
static hipError_t launch_qs(const uint16_t* x, int64_t rows, int64_t K, int64_t k_stride, uint8_t* codes,
                            uint8_t* scales, hipStream_t s) {
  hipLaunchKernelGGL((quantize_strided_kernel<SK, ASYM>), dim3((unsigned)((rows + 255) / 256), (unsigned)(K / 32)),
                     dim3(256), 0, s, x, rows, K, k_stride, codes, scales);
  return hipGetLastError();
}

hipError_t launch_quantize_strided(int scale_kind, bool asym, const uint16_t* x, int64_t rows, int64_t K,
                                   int64_t k_stride, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  switch (scale_kind) {
    case kScaleE5M2:
      return asym ? launch_qs<kScaleE5M2, true>(x, rows, K, k_stride, codes, scales, s)
                  : launch_qs<kScaleE5M2, false>(x, rows, K, k_stride, codes, scales, s);
    case kScaleE8M0Floor:
      return asym ? launch_qs<kScaleE8M0Floor, true>(x, rows, K, k_stride, codes, scales, s)
                  : launch_qs<kScaleE8M0Floor, false>(x, rows, K, k_stride, codes, scales, s);
    case kScaleE8M0Round:
      return asym ? launch_qs<kScaleE8M0Round, true>(x, rows, K, k_stride, codes, scales, s)
                  : launch_qs<kScaleE8M0Round, false>(x, rows, K, k_stride, codes, scales, s);
  }
  return hipErrorInvalidValue;
}

template <int SK, bool ASYM>
static hipError_t launch_dq(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K, void* out,
                            int out_dtype, hipStream_t s) {
  const dim3 grid(grid_for(rows * (K / 8)));
  if (out_dtype == 1)
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, true>), grid, dim3(256), 0, s, codes, scales, rows, K, out);
  else
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, false>), grid, dim3(256), 0, s, codes, scales, rows, K, out);
  return hipGetLastError();
}

hipError_t launch_dequantize(int scale_kind, bool asym, const uint8_t* codes, const uint8_t* scales, int64_t rows,
                             int64_t K, void* out, int out_dtype, hipStream_t s) {
  // E8M0 floor and round share the byte encoding
  if (scale_kind == kScaleE5M2)
    return asym ? launch_dq<kScaleE5M2, true>(codes, scales, rows, K, out, out_dtype, s)
                : launch_dq<kScaleE5M2, false>(codes, scales, rows, K, out, out_dtype, s);
  return asym ? launch_dq<kScaleE8M0Floor, true>(codes, scales, rows, K, out, out_dtype, s)
              : launch_dq<kScaleE8M0Floor, false>(codes, scales, rows, K, out, out_dtype, s);
}

}  // namespace amx
