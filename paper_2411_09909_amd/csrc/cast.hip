// Direct-cast quantization BF16 -> AMXFP4 / MXFP4 (Appendix B Algorithm 1, generalised by Sec. 4.2 Eq. 1 to a
// sign-dependent pair of shared scales) and the matching dequantization (Eq. 1). Group sizes 16, 32, 64, 128 along K
// (Sec. 5.3 / Table 5 compare them; 32 is the paper's choice); scale formats FP8 E5M2 (the paper's), FP8 E4M3 and
// E8M0 with the exponent floored or rounded; optionally a tensor-wise FP32 scale underneath (Sec. 5.3, the double
// scaling of NVFP4 / ANVFP4): elements are multiplied by its reciprocal in FP32 first and the cast runs on those.
//
// Contiguous cast: one lane owns 16 consecutive BF16 (two 128-bit loads); the GS / 16 lanes next to each other own
// one group. Group extrema are found with packed 16-bit integer max (non-negative BF16 patterns order like integers)
// and DPP permutes inside the group. Every decision comes out as exact arithmetic would give it. For BF16 elements
// (the plain cast) a value that is not on a rounding boundary is at least 2^-9 of it away, which cheap arithmetic
// resolves (the BF16 section of cast_math.h): scale = hardware FP8 conversion of amax * fl(1/6) snapped to 13 bits,
// element = x * rcp(scale) rounded to binary16 and then to E2M1 by v_cvt_scalef32_pk_fp4_f16. For FP32 elements (a
// tensor-wise scale underneath; values computed by another kernel) the general forms are used:
//   - an FP8 scale is the correctly rounded FP32 quotient amax/6 rounded once more to 3 (E5M2) or 4 (E4M3)
//     significant bits, which equals rounding the real quotient (see fp8_scale());
//   - the element quotient x / S is formed correctly rounded away from FP32 midpoints and exactly when representable,
//     which keeps it on the right side of every E2M1 boundary (see quotient()), and rounded to E2M1 by the hardware
//     conversion v_cvt_scalef32_pk_fp4_f32.
// Strided cast (groups down a column, for V in P.V): one lane per (row, group), the same arithmetic.
// Whole-row groups (group size -1, as in the code example of Appendix B): one thread block per row, two sweeps.
#include "cast_core.h"
#include "device_formats.h"

namespace amx {

// Eight values (the class of each is its sign bit) -> eight E2M1 codes, first element in the lowest nibble. The E2M1
// rounding itself (nearest, ties to even, saturating, sign kept on zero results) is done by the packed FP32 -> FP4
// conversion instruction.
template <int SCALE_KIND, bool ASYM>
__device__ __forceinline__ uint32_t encode8(const float (&y)[8], float s_pos, float r_pos, float s_neg, float r_neg) {
  uint32_t packed = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float x0 = y[2 * j], x1 = y[2 * j + 1];
    float z0, z1;
    if constexpr (ASYM) {
      const bool n0 = (int32_t)f2u(x0) < 0, n1 = (int32_t)f2u(x1) < 0;
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

// Largest magnitude per sign class over n floats, as bit patterns (non-negative floats order like integers).
// Symmetric formats: both results are the largest magnitude overall.
template <bool ASYM, int N>
__device__ __forceinline__ void class_extrema(const float (&y)[N], uint32_t& amax_p, uint32_t& amax_n) {
  amax_p = 0, amax_n = 0;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const uint32_t bits = f2u(y[i]), mag = bits & 0x7FFFFFFFu;
    if (ASYM && (bits >> 31))
      amax_n = mag > amax_n ? mag : amax_n;
    else
      amax_p = mag > amax_p ? mag : amax_p;
  }
  if constexpr (!ASYM) amax_n = amax_p;
}

// Contiguous cast. One lane owns 16 consecutive BF16 (two 128-bit loads, one 64-bit store of codes). Thread block =
// 256 lanes arranged as (256 >> bx_log2) rows x (1 << bx_log2) chunks of 16 elements; blockIdx.x walks the rows,
// blockIdx.y the chunks of a row. A group is 2^lpg_log2 neighbouring lanes (1 lane for groups of 16 ... 8 lanes for
// groups of 128); bx is a multiple of that and so is the number of chunks in a row, hence a group is always whole
// and aligned in its wave.
// TENSOR_SCALED (Sec. 5.3, double scaling): every element is first multiplied by the tensor-wise factor
// tensor_pair[1] in FP32 (one rounding) and the group-wise cast runs on those FP32 values.
// ONE_ROW: the launcher chose bx_log2 = 8 (a row has at least 256 chunks), so a thread block lies in one row and all
// row arithmetic is uniform (scalar unit).
template <int SCALE_KIND, bool ASYM, bool TENSOR_SCALED, bool ONE_ROW>
__global__ __launch_bounds__(256) void quantize_contig_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                              int64_t row_stride, int64_t batch_stride,
                                                              const float* __restrict__ tensor_pair,
                                                              uint8_t* __restrict__ codes,
                                                              uint8_t* __restrict__ scales, int bx_log2,
                                                              int lpg_log2) {
  // blockIdx.z: batch entry (operands batch_stride elements apart; outputs packed one after the other)
  x += (int64_t)blockIdx.z * batch_stride;
  codes += (int64_t)blockIdx.z * rows * (K >> 1);
  scales += (int64_t)blockIdx.z * rows * (K >> (lpg_log2 + 4)) * (ASYM ? 2 : 1);
  const int tx = ONE_ROW ? (int)threadIdx.x : (int)threadIdx.x & ((1 << bx_log2) - 1);
  const int ty = ONE_ROW ? 0 : (int)threadIdx.x >> bx_log2;
  const int64_t r = ONE_ROW ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * (256 >> bx_log2) + ty;
  const int cc = (int)(blockIdx.y << (ONE_ROW ? 8 : bx_log2)) + tx;  // chunk of 16 elements within the row
  if (r >= rows || cc >= (int)(K >> 4)) return;
  const uint4* src = reinterpret_cast<const uint4*>(x + r * row_stride + (int64_t)cc * 16);
  const uint4 v0 = src[0], v1 = src[1];
  const uint32_t d[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
  uint32_t code_lo, code_hi, sb_p, sb_n;
  if constexpr (TENSOR_SCALED) {
    float y[16];
#pragma unroll
    for (int j = 0; j < 8; ++j) y[2 * j] = u2f(d[j] << 16), y[2 * j + 1] = u2f(d[j] & 0xFFFF0000u);
    const float rt = tensor_pair[1];
#pragma unroll
    for (int i = 0; i < 16; ++i) y[i] *= rt;
    // group extrema (steps "max_i |V_i|" of Algorithm 1, split by sign for the asymmetric format)
    uint32_t amax_p, amax_n;
    class_extrema<ASYM>(y, amax_p, amax_n);
    amax_p = group_max_u32(amax_p, lpg_log2);
    if constexpr (ASYM) amax_n = group_max_u32(amax_n, lpg_log2);
    float s_pos, r_pos, s_neg, r_neg;
    sb_p = encode_scale_sr<SCALE_KIND>(u2f(amax_p), s_pos, r_pos);
    sb_n = sb_p, s_neg = s_pos, r_neg = r_pos;
    if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(u2f(amax_n), s_neg, r_neg);
    const float ylo[8] = {y[0], y[1], y[2], y[3], y[4], y[5], y[6], y[7]};
    const float yhi[8] = {y[8], y[9], y[10], y[11], y[12], y[13], y[14], y[15]};
    code_lo = encode8<SCALE_KIND, ASYM>(ylo, s_pos, r_pos, s_neg, r_neg);
    code_hi = encode8<SCALE_KIND, ASYM>(yhi, s_pos, r_pos, s_neg, r_neg);
  } else {
    uint32_t code[2];
    cast_words_bf16<SCALE_KIND, ASYM, 16>(d, lpg_log2, code, sb_p, sb_n);
    code_lo = code[0], code_hi = code[1];
  }
  *reinterpret_cast<uint2*>(codes + r * (K >> 1) + (int64_t)cc * 8) = make_uint2(code_lo, code_hi);
  if ((tx & ((1 << lpg_log2) - 1)) == 0) {
    const int64_t g = r * (K >> (lpg_log2 + 4)) + (cc >> lpg_log2);
    if constexpr (ASYM)
      *reinterpret_cast<uint16_t*>(scales + g * 2) = (uint16_t)(sb_p | (sb_n << 8));
    else
      scales[g] = (uint8_t)sb_p;
  }
}

// One group per row (the code example of Appendix B casts its tensor this way). One thread block per (row, batch
// entry); a lane owns the 8-element chunks threadIdx.x, threadIdx.x + blockDim.x, ... of the row. First sweep: per
// class extrema of the lane's chunks, reduced over the wave with lane exchanges and over the block's waves through
// LDS. Second sweep (the row then comes from the cache): the element step of the grouped casts with the row's
// scale(s). TENSOR_SCALED as in quantize_contig_kernel.
template <int SCALE_KIND, bool ASYM, bool TENSOR_SCALED>
__global__ __launch_bounds__(256) void quantize_row_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                           int64_t row_stride, int64_t batch_stride,
                                                           const float* __restrict__ tensor_pair,
                                                           uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
  __shared__ uint32_t wave_max[2][4];
  const int64_t r = blockIdx.x, out_row = (int64_t)blockIdx.y * rows + r;
  const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)blockIdx.y * batch_stride + r * row_stride);
  const int chunks = (int)(K >> 3), lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  float rt = 1.0f;
  if constexpr (TENSOR_SCALED) rt = tensor_pair[1];
  // largest magnitude per sign class, as FP32 bit patterns (non-negative floats order like integers)
  uint32_t amax_p = 0, amax_n = 0;
  for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
    const uint4 v = src[c];
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    float y[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) y[2 * j] = u2f(d[j] << 16) * rt, y[2 * j + 1] = u2f(d[j] & 0xFFFF0000u) * rt;
    uint32_t p, n;
    class_extrema<ASYM>(y, p, n);
    amax_p = p > amax_p ? p : amax_p;
    amax_n = n > amax_n ? n : amax_n;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t p = __shfl_xor(amax_p, o), n = __shfl_xor(amax_n, o);
    amax_p = p > amax_p ? p : amax_p;
    amax_n = n > amax_n ? n : amax_n;
  }
  if (lane == 0) wave_max[0][wave] = amax_p, wave_max[1][wave] = amax_n;
  __syncthreads();
  for (int w = 0; w < waves; ++w) {
    const uint32_t p = wave_max[0][w], n = wave_max[1][w];
    amax_p = p > amax_p ? p : amax_p;
    amax_n = n > amax_n ? n : amax_n;
  }
  float s_pos = 0.f, r_pos, s_neg = 0.f, r_neg;
  uint32_t sb_p, sb_n;
  if constexpr (TENSOR_SCALED) {
    sb_p = encode_scale_sr<SCALE_KIND>(u2f(amax_p), s_pos, r_pos);
    sb_n = sb_p, s_neg = s_pos, r_neg = r_pos;
    if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(u2f(amax_n), s_neg, r_neg);
  } else {
    sb_p = encode_scale_r_bf16<SCALE_KIND>(u2f(amax_p), r_pos);
    sb_n = sb_p, r_neg = r_pos;
    if constexpr (ASYM) sb_n = encode_scale_r_bf16<SCALE_KIND>(u2f(amax_n), r_neg);
  }
  if (threadIdx.x == 0) {
    if constexpr (ASYM)
      scales[out_row * 2] = (uint8_t)sb_p, scales[out_row * 2 + 1] = (uint8_t)sb_n;
    else
      scales[out_row] = (uint8_t)sb_p;
  }
  uint32_t* dst = reinterpret_cast<uint32_t*>(codes + out_row * (K >> 1));
  for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
    const uint4 v = src[c];
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    if constexpr (TENSOR_SCALED) {
      float y[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) y[2 * j] = u2f(d[j] << 16) * rt, y[2 * j + 1] = u2f(d[j] & 0xFFFF0000u) * rt;
      dst[c] = encode8<SCALE_KIND, ASYM>(y, s_pos, r_pos, s_neg, r_neg);
    } else {
      dst[c] = encode8_bf16<ASYM>(d, r_pos, r_neg);
    }
  }
}

// Groups run down a column: element (r, k) = x[r + k * k_stride]. One lane owns one (row, group) of GS elements;
// consecutive lanes own consecutive rows, so each of the GS loads of a wave reads 128 contiguous bytes.
// grid: (K / GS groups, ceil(rows / 256), batch).
template <int SCALE_KIND, bool ASYM, bool TENSOR_SCALED, int GS>
__global__ __launch_bounds__(256) void quantize_strided_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                               int64_t k_stride, int64_t batch_stride,
                                                               const float* __restrict__ tensor_pair,
                                                               uint8_t* __restrict__ codes,
                                                               uint8_t* __restrict__ scales) {
  const int64_t G = K / GS;
  x += (int64_t)blockIdx.z * batch_stride;
  codes += (int64_t)blockIdx.z * rows * (K >> 1);
  scales += (int64_t)blockIdx.z * rows * G * (ASYM ? 2 : 1);
  const int64_t r = (int64_t)blockIdx.y * 256 + threadIdx.x;
  const int64_t g = blockIdx.x;
  if (r >= rows) return;
  const uint16_t* p = x + r + g * GS * k_stride;
  float rt = 1.0f;
  if constexpr (TENSOR_SCALED) rt = tensor_pair[1];
  float y[GS];
#pragma unroll
  for (int i = 0; i < GS; ++i) {
    y[i] = u2f((uint32_t)p[i * k_stride] << 16);
    if constexpr (TENSOR_SCALED) y[i] *= rt;
  }
  uint32_t amax_p, amax_n;
  class_extrema<ASYM>(y, amax_p, amax_n);
  float s_pos, r_pos, s_neg, r_neg;
  const uint32_t sb_p = encode_scale_sr<SCALE_KIND>(u2f(amax_p), s_pos, r_pos);
  uint32_t sb_n = sb_p;
  s_neg = s_pos, r_neg = r_pos;
  if constexpr (ASYM) sb_n = encode_scale_sr<SCALE_KIND>(u2f(amax_n), s_neg, r_neg);
  uint32_t* out = reinterpret_cast<uint32_t*>(codes + r * (K >> 1) + g * (GS / 2));
#pragma unroll
  for (int t = 0; t < GS / 16; ++t) {
    const float lo[8] = {y[16 * t], y[16 * t + 1], y[16 * t + 2], y[16 * t + 3],
                         y[16 * t + 4], y[16 * t + 5], y[16 * t + 6], y[16 * t + 7]};
    const float hi[8] = {y[16 * t + 8], y[16 * t + 9], y[16 * t + 10], y[16 * t + 11],
                         y[16 * t + 12], y[16 * t + 13], y[16 * t + 14], y[16 * t + 15]};
    *reinterpret_cast<uint2*>(out + 2 * t) =
        make_uint2(encode8<SCALE_KIND, ASYM>(lo, s_pos, r_pos, s_neg, r_neg),
                   encode8<SCALE_KIND, ASYM>(hi, s_pos, r_pos, s_neg, r_neg));
  }
  if constexpr (ASYM)
    *reinterpret_cast<uint16_t*>(scales + (r * G + g) * 2) = (uint16_t)(sb_p | (sb_n << 8));
  else
    scales[r * G + g] = (uint8_t)sb_p;
}

// Tensor-wise scale (Sec. 5.3, double scaling): the largest magnitude of a BF16 tensor, then
// S_t = amax / 2688 (2688 = 448 * 6 = largest E4M3 group scale times largest element), not below 2^-96, and
// R_t = 1 / S_t, both correctly rounded FP32 divisions; an all-zero tensor gives 1, 1. pair[0] serves as the
// accumulator of the maximum (bit pattern of a non-negative float) between the three launches.
__global__ void tensor_amax_init_kernel(uint32_t* pair) {
  pair[0] = 0u;
  pair[1] = 0u;
}

__global__ __launch_bounds__(256) void tensor_amax_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t K,
                                                          int64_t row_stride, uint32_t* __restrict__ pair) {
  const int64_t chunks_per_row = K >> 3, total = rows * chunks_per_row;
  uint32_t m = 0;  // two running 15-bit magnitudes
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < total; c += (int64_t)gridDim.x * 256) {
    const int64_t r = c / chunks_per_row, cc = c - r * chunks_per_row;
    const uint4 v = *reinterpret_cast<const uint4*>(x + r * row_stride + cc * 8);
    m = pk_max_i16(m, pk_max_i16(pk_max_i16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                                 pk_max_i16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu)));
  }
  uint32_t a = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)a, off, 64);
    a = a > o ? a : o;
  }
  // one atomic per workgroup, and none when the running maximum already covers it (the maximum only grows, so a
  // stale read can only cause a superfluous atomic)
  __shared__ uint32_t wave_max[4];
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) a = a > wave_max[w] ? a : wave_max[w];
    a <<= 16;
    if (a > __builtin_nontemporal_load(pair)) atomicMax(pair, a);
  }
}

__global__ void tensor_scale_finalize_kernel(float* pair) {
  const float amax = pair[0];  // the accumulated bit pattern is the float itself
  float st = 1.0f, rt = 1.0f;
  if (amax > 0.f) {
    st = fmaxf(__fdiv_rn(amax, 2688.0f), 0x1p-96f);
    rt = __fdiv_rn(1.0f, st);
  }
  pair[0] = st;
  pair[1] = rt;
}

// x_hat = (-1)^s * elem * S_class (Eq. 1), times the tensor-wise scale tensor_pair[0] when that pointer is not null
// (Sec. 5.3; FP32 output only: one rounding of the exact product). One lane expands 8 codes.
template <int SCALE_KIND, bool ASYM, bool OUT_BF16>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t* __restrict__ codes,
                                                         const uint8_t* __restrict__ scales, int64_t rows, int64_t K,
                                                         int gs_log2, const float* __restrict__ tensor_pair,
                                                         void* __restrict__ out) {
  const float st = tensor_pair ? tensor_pair[0] : 1.0f;
  const int64_t chunks_per_row = K >> 3;
  const int64_t total = rows * chunks_per_row;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < total; c += (int64_t)gridDim.x * 256) {
    const int64_t r = c / chunks_per_row;
    const int64_t cc = c - r * chunks_per_row;
    const uint32_t w = *reinterpret_cast<const uint32_t*>(codes + r * (K >> 1) + cc * 4);
    const int64_t g = r * groups_per_row(K, gs_log2) + ((cc * 8) >> gs_log2);
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
      v[j] = (mag2 * s) * st;  // elem * scale has <= 6 significant bits: exact in FP32 and in BF16
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
static hipError_t launch_qc(const uint16_t* x, int64_t rows, int64_t K, int gs_log2, int64_t row_stride,
                            int64_t batch, int64_t batch_stride, const float* tensor_pair, uint8_t* codes,
                            uint8_t* scales, hipStream_t s) {
  // block shape: as many chunks of a row as fit (power of two, one group .. 256), the rest of the 256 lanes go to
  // more rows
  const int64_t chunks = K / 16;
  const int lpg_log2 = gs_log2 - 4;
  int bx_log2 = lpg_log2;
  while (bx_log2 < 8 && (int64_t(1) << (bx_log2 + 1)) <= chunks) ++bx_log2;
  const int64_t bx = int64_t(1) << bx_log2, by = 256 >> bx_log2;
  const dim3 grid((unsigned)((rows + by - 1) / by), (unsigned)((chunks + bx - 1) / bx), (unsigned)batch);
  auto launch = [&]<bool SCALED, bool ONE_ROW>() {
    hipLaunchKernelGGL((quantize_contig_kernel<SK, ASYM, SCALED, ONE_ROW>), grid, dim3(256), 0, s, x, rows, K,
                       row_stride, batch_stride, tensor_pair, codes, scales, bx_log2, lpg_log2);
  };
  if (tensor_pair)
    bx_log2 == 8 ? launch.template operator()<true, true>() : launch.template operator()<true, false>();
  else
    bx_log2 == 8 ? launch.template operator()<false, true>() : launch.template operator()<false, false>();
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
                                  int64_t K, int64_t row_stride, int64_t batch, int64_t batch_stride,
                                  const float* tensor_pair, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || !group_divides(K, group_size)) return hipErrorInvalidValue;
  if (gl == kWholeRowLog2) {
    // one wave per short row (up to 8 chunks a lane), four waves beyond
    const dim3 grid((unsigned)rows, (unsigned)batch), block(K <= 4096 ? 64 : 256);
    return for_format(scale_kind, asym, [&]<int SK, bool ASYM>() {
      if (tensor_pair)
        hipLaunchKernelGGL((quantize_row_kernel<SK, ASYM, true>), grid, block, 0, s, x, rows, K, row_stride,
                           batch_stride, tensor_pair, codes, scales);
      else
        hipLaunchKernelGGL((quantize_row_kernel<SK, ASYM, false>), grid, block, 0, s, x, rows, K, row_stride,
                           batch_stride, tensor_pair, codes, scales);
      return hipGetLastError();
    });
  }
  return for_format(scale_kind, asym, [&]<int SK, bool ASYM>() {
    return launch_qc<SK, ASYM>(x, rows, K, gl, row_stride, batch, batch_stride, tensor_pair, codes, scales, s);
  });
}

template <int SK, bool ASYM, int GS>
static hipError_t launch_qs(const uint16_t* x, int64_t rows, int64_t K, int64_t k_stride, int64_t batch,
                            int64_t batch_stride, const float* tensor_pair, uint8_t* codes, uint8_t* scales,
                            hipStream_t s) {
  const dim3 grid((unsigned)(K / GS), (unsigned)((rows + 255) / 256), (unsigned)batch);
  if (tensor_pair)
    hipLaunchKernelGGL((quantize_strided_kernel<SK, ASYM, true, GS>), grid, dim3(256), 0, s, x, rows, K, k_stride,
                       batch_stride, tensor_pair, codes, scales);
  else
    hipLaunchKernelGGL((quantize_strided_kernel<SK, ASYM, false, GS>), grid, dim3(256), 0, s, x, rows, K, k_stride,
                       batch_stride, tensor_pair, codes, scales);
  return hipGetLastError();
}

hipError_t launch_quantize_strided(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, int64_t rows,
                                   int64_t K, int64_t k_stride, int64_t batch, int64_t batch_stride,
                                   const float* tensor_pair, uint8_t* codes, uint8_t* scales, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || gl == kWholeRowLog2 || K % group_size != 0) return hipErrorInvalidValue;
  return for_format(scale_kind, asym, [&]<int SK, bool ASYM>() {
    switch (gl) {
      case 4: return launch_qs<SK, ASYM, 16>(x, rows, K, k_stride, batch, batch_stride, tensor_pair, codes, scales, s);
      case 5: return launch_qs<SK, ASYM, 32>(x, rows, K, k_stride, batch, batch_stride, tensor_pair, codes, scales, s);
      case 6: return launch_qs<SK, ASYM, 64>(x, rows, K, k_stride, batch, batch_stride, tensor_pair, codes, scales, s);
      default: return launch_qs<SK, ASYM, 128>(x, rows, K, k_stride, batch, batch_stride, tensor_pair, codes, scales, s);
    }
  });
}

template <int SK, bool ASYM>
static hipError_t launch_dq(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K, int gs_log2,
                            const float* tensor_pair, void* out, int out_dtype, hipStream_t s) {
  const dim3 grid(grid_for(rows * (K / 8)));
  if (out_dtype == 1)
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, true>), grid, dim3(256), 0, s, codes, scales, rows, K, gs_log2,
                       tensor_pair, out);
  else
    hipLaunchKernelGGL((dequantize_kernel<SK, ASYM, false>), grid, dim3(256), 0, s, codes, scales, rows, K, gs_log2,
                       tensor_pair, out);
  return hipGetLastError();
}

hipError_t launch_dequantize(int scale_kind, bool asym, int64_t group_size, const uint8_t* codes,
                             const uint8_t* scales, int64_t rows, int64_t K, const float* tensor_pair, void* out,
                             int out_dtype, hipStream_t s) {
  const int gl = group_log2(group_size);
  if (gl < 0 || !group_divides(K, group_size)) return hipErrorInvalidValue;
  // E8M0 floor and round share the byte encoding
  return for_format(scale_kind == kScaleE8M0Round ? kScaleE8M0Floor : scale_kind, asym, [&]<int SK, bool ASYM>() {
    return launch_dq<SK, ASYM>(codes, scales, rows, K, gl, tensor_pair, out, out_dtype, s);
  });
}

hipError_t launch_tensor_scale(const uint16_t* x, int64_t rows, int64_t K, int64_t row_stride, float* pair,
                               hipStream_t s) {
  uint32_t* acc = reinterpret_cast<uint32_t*>(pair);
  hipLaunchKernelGGL(tensor_amax_init_kernel, dim3(1), dim3(1), 0, s, acc);
  // 8 workgroups per CU, grid-stride: few atomics on the one accumulator
  const int amax_blocks = grid_for(rows * (K / 8)) < 2048 ? grid_for(rows * (K / 8)) : 2048;
  hipLaunchKernelGGL(tensor_amax_kernel, dim3(amax_blocks), dim3(256), 0, s, x, rows, K, row_stride, acc);
  hipLaunchKernelGGL(tensor_scale_finalize_kernel, dim3(1), dim3(1), 0, s, pair);
  return hipGetLastError();
}

}  // namespace amx
