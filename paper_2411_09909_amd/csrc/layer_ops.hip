// Glue operators of the decoder-layer workload (include/amxfp4_layer.h): the BF16 operators that sit between the
// quantized matrix multiplications of a LLaMA-style layer (Sec. 5.1 evaluates with every matmul of the decoder layers
// quantized and everything else left in BF16). All of them are memory-bound elementwise or row-wise kernels: FP32 (or
// BF16) in, BF16 out, FP32 arithmetic, 128-bit accesses.
#include "../../include/amxfp4.h"
#include "../../include/amxfp4_layer.h"
#include "cast_core.h"
#include "device_formats.h"
#include "kernels.h"
#include "layer_math.h"

namespace amx {
namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// reduction over the 256 threads of a block (4 waves); every thread gets the result
template <bool MAX>
__device__ __forceinline__ float block_reduce(float v, float* smem) {
  v = MAX ? wave_max(v) : wave_sum(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();  // smem may still be read from a previous reduction
  if ((threadIdx.x & 63) == 0) smem[wave] = v;
  __syncthreads();
  const float a = smem[0], b = smem[1], c = smem[2], d = smem[3];
  return MAX ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

// one block per row; a thread holds up to kMaxChunks runs of 8 elements
constexpr int kRmsMaxChunks = 8;  // 256 threads x 8 x 8 = 16384 elements
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint16_t* __restrict__ x, const float* __restrict__ w,
                                                      int64_t dim, float eps, uint16_t* __restrict__ out) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const int chunks = (int)(dim >> 3);
  float v[kRmsMaxChunks][8];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < kRmsMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks) {
      const uint4 u = *reinterpret_cast<const uint4*>(x + row * dim + (int64_t)ci * 8);
      const uint32_t d[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[c][2 * j] = u2f(d[j] << 16);
        v[c][2 * j + 1] = u2f(d[j] & 0xFFFF0000u);
        ss += v[c][2 * j] * v[c][2 * j] + v[c][2 * j + 1] * v[c][2 * j + 1];
      }
    }
  }
  ss = block_reduce<false>(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)dim + eps);
#pragma unroll
  for (int c = 0; c < kRmsMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks) {
      const float4 w0 = *reinterpret_cast<const float4*>(w + (int64_t)ci * 8);
      const float4 w1 = *reinterpret_cast<const float4*>(w + (int64_t)ci * 8 + 4);
      const float ww[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = pack2(v[c][2 * j] * inv * ww[2 * j], v[c][2 * j + 1] * inv * ww[2 * j + 1]);
      *reinterpret_cast<uint4*>(out + row * dim + (int64_t)ci * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// rmsnorm_kernel with the cast of its result fused in (and, with ADD, the residual addition in front of it): the
// element-to-lane mapping, the order of the sum of squares and every rounding are those of residual_add_kernel and
// rmsnorm_kernel, so the BF16 row that is cast here, in registers, is bit for bit the row those two kernels would
// have written, and the codes and scales are what amxfp4_quantize makes of it (cast_core.h). A group of the cast is
// 2^lanes_log2 neighbouring lanes of 8 elements each; dim is a multiple of the group size, so the lanes of a group
// are all inside the row or all outside.
// (x and sum_out are not declared restrict: they may be the same buffer, each lane reads its elements before it writes
// them and nobody else touches them)
template <int SCALE_KIND, bool ASYM, bool ADD>
__global__ __launch_bounds__(256) void rmsnorm_quantize_kernel(const uint16_t* x, const float* __restrict__ y,
                                                               uint16_t* sum_out,
                                                               const float* __restrict__ w, int64_t dim, float eps,
                                                               int lanes_log2, uint8_t* __restrict__ codes,
                                                               uint8_t* __restrict__ scales) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const int chunks = (int)(dim >> 3);
  float v[kRmsMaxChunks][8];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < kRmsMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks) {
      const uint4 u = *reinterpret_cast<const uint4*>(x + row * dim + (int64_t)ci * 8);
      uint32_t d[4] = {u.x, u.y, u.z, u.w};
      if constexpr (ADD) {
        const float4 y0 = *reinterpret_cast<const float4*>(y + row * dim + (int64_t)ci * 8);
        const float4 y1 = *reinterpret_cast<const float4*>(y + row * dim + (int64_t)ci * 8 + 4);
        const float yy[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
          d[j] = pack2(u2f(d[j] << 16) + yy[2 * j], u2f(d[j] & 0xFFFF0000u) + yy[2 * j + 1]);
        *reinterpret_cast<uint4*>(sum_out + row * dim + (int64_t)ci * 8) = make_uint4(d[0], d[1], d[2], d[3]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[c][2 * j] = u2f(d[j] << 16);
        v[c][2 * j + 1] = u2f(d[j] & 0xFFFF0000u);
        ss += v[c][2 * j] * v[c][2 * j] + v[c][2 * j + 1] * v[c][2 * j + 1];
      }
    }
  }
  ss = block_reduce<false>(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)dim + eps);
  const int64_t groups_per_row = dim >> (lanes_log2 + 3);
#pragma unroll
  for (int c = 0; c < kRmsMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks) {
      const float4 w0 = *reinterpret_cast<const float4*>(w + (int64_t)ci * 8);
      const float4 w1 = *reinterpret_cast<const float4*>(w + (int64_t)ci * 8 + 4);
      const float ww[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = pack2(v[c][2 * j] * inv * ww[2 * j], v[c][2 * j + 1] * inv * ww[2 * j + 1]);
      uint32_t code[1], sb_p, sb_n;
      cast_words_bf16<SCALE_KIND, ASYM, 8>(o, lanes_log2, code, sb_p, sb_n);
      *reinterpret_cast<uint32_t*>(codes + row * (dim >> 1) + (int64_t)ci * 4) = code[0];
      if ((threadIdx.x & ((1 << lanes_log2) - 1)) == 0) {
        const int64_t g = row * groups_per_row + (ci >> lanes_log2);
        if constexpr (ASYM)
          *reinterpret_cast<uint16_t*>(scales + g * 2) = (uint16_t)(sb_p | (sb_n << 8));
        else
          scales[g] = (uint8_t)sb_p;
      }
    }
  }
}

// One thread per (token, pair i < head_dim / 2) and chunk of kRopeHeads heads (blockIdx.y): the angle of a pair does
// not depend on the head, so its FP64 sine and cosine are computed once per thread and reused for the chunk.
constexpr int kRopeHeads = 8;
__global__ __launch_bounds__(256) void split_heads_rope_kernel(const float* __restrict__ in, int64_t seq, int64_t ld,
                                                               int64_t col0, int64_t heads, int half, int rotate,
                                                               int64_t pos0, double log_theta,
                                                               uint16_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= seq * half) return;
  const int i = (int)(idx % half);
  const int64_t s = idx / half;
  double sn = 0.0, cs = 1.0;
  if (rotate) {
    // angle = pos * theta^(-2 i / head_dim), in FP64 so that it does not depend on how the power is evaluated
    const double ang = (double)(pos0 + s) * exp(-log_theta * (double)i / (double)half);
    sincos(ang, &sn, &cs);
  }
  const int64_t h0 = (int64_t)blockIdx.y * kRopeHeads, h1 = h0 + kRopeHeads < heads ? h0 + kRopeHeads : heads;
  for (int64_t h = h0; h < h1; ++h) {
    const float* p = in + s * ld + col0 + h * 2 * half;
    const float x1 = p[i], x2 = p[i + half];
    float o1 = x1, o2 = x2;
    if (rotate) {
      o1 = (float)((double)x1 * cs - (double)x2 * sn);
      o2 = (float)((double)x2 * cs + (double)x1 * sn);
    }
    uint16_t* q = out + (h * seq + s) * 2 * half;
    q[i] = (uint16_t)bf16_rne(o1);
    q[i + half] = (uint16_t)bf16_rne(o2);
  }
}

// split_heads_rope_kernel (rotate) followed by the cast of its result along the head dimension, in one pass: the
// rotated BF16 heads are never written. One thread per (token, run of 8 dimensions d0 .. d0 + 7 below head_dim / 2)
// and chunk of kRopeHeads heads: it forms the 8 outputs at d0 .. and the 8 at d0 + head_dim / 2 .. (they share their
// angles), each run is one lane's share of a group of 32, and the four neighbouring threads of a group exchange their
// extrema as the cast kernel's lanes do (cast_core.h). head_dim % 64 == 0, so a group never straddles the two halves
// and the threads of a token are a whole number of quads. Same arithmetic as the two separate kernels: same bits.
template <int SCALE_KIND, bool ASYM>
__global__ __launch_bounds__(256) void rope_quantize_kernel(const float* __restrict__ in, int64_t seq, int64_t ld,
                                                            int64_t col0, int64_t heads, int half, int64_t pos0,
                                                            double log_theta, uint8_t* __restrict__ codes,
                                                            uint8_t* __restrict__ scales) {
  const int runs = half >> 3;  // threads per token
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= seq * runs) return;  // (whole quads: seq * runs is a multiple of 4)
  const int j = (int)(idx % runs);
  const int64_t s = idx / runs;
  double sn[8], cs[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double ang = (double)(pos0 + s) * exp(-log_theta * (double)(8 * j + e) / (double)half);
    sincos(ang, &sn[e], &cs[e]);
  }
  const int groups = half >> 4;  // groups of 32 per head
  const int64_t h0 = (int64_t)blockIdx.y * kRopeHeads, h1 = h0 + kRopeHeads < heads ? h0 + kRopeHeads : heads;
  for (int64_t h = h0; h < h1; ++h) {
    const float* p = in + s * ld + col0 + h * 2 * half + 8 * j;
    const float4 a0 = *reinterpret_cast<const float4*>(p), a1 = *reinterpret_cast<const float4*>(p + 4);
    const float4 b0 = *reinterpret_cast<const float4*>(p + half), b1 = *reinterpret_cast<const float4*>(p + half + 4);
    const float x1[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    const float x2[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    float o1[8], o2[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o1[e] = (float)((double)x1[e] * cs[e] - (double)x2[e] * sn[e]);
      o2[e] = (float)((double)x2[e] * cs[e] + (double)x1[e] * sn[e]);
    }
    const uint32_t d1[4] = {pack2(o1[0], o1[1]), pack2(o1[2], o1[3]), pack2(o1[4], o1[5]), pack2(o1[6], o1[7])};
    const uint32_t d2[4] = {pack2(o2[0], o2[1]), pack2(o2[2], o2[3]), pack2(o2[4], o2[5]), pack2(o2[6], o2[7])};
    uint32_t c1[1], c2[1], p1, n1, p2, n2;
    cast_words_bf16<SCALE_KIND, ASYM, 8>(d1, 2, c1, p1, n1);
    cast_words_bf16<SCALE_KIND, ASYM, 8>(d2, 2, c2, p2, n2);
    const int64_t row = h * seq + s;
    uint8_t* crow = codes + row * half;  // head_dim / 2 bytes of codes per row
    *reinterpret_cast<uint32_t*>(crow + 4 * j) = c1[0];
    *reinterpret_cast<uint32_t*>(crow + (half >> 1) + 4 * j) = c2[0];
    if ((j & 3) == 0) {
      const int64_t g1 = row * groups + (j >> 2), g2 = g1 + (groups >> 1);
      if constexpr (ASYM) {
        *reinterpret_cast<uint16_t*>(scales + g1 * 2) = (uint16_t)(p1 | (n1 << 8));
        *reinterpret_cast<uint16_t*>(scales + g2 * 2) = (uint16_t)(p2 | (n2 << 8));
      } else {
        scales[g1] = (uint8_t)p1;
        scales[g2] = (uint8_t)p2;
      }
    }
  }
}

// one block per score row; a thread holds up to kSmMaxChunks runs of 8 columns
constexpr int kSmMaxChunks = 8;  // 16384 columns
__global__ __launch_bounds__(256) void softmax_causal_kernel(const float* __restrict__ s, int64_t rows, int64_t cols,
                                                             float scale, uint16_t* __restrict__ out) {
  __shared__ float red[4];
  const int64_t r = blockIdx.x;             // row within the batch entry
  const int64_t base = ((int64_t)blockIdx.y * rows + r) * cols;
  const int last = (int)(r % cols);         // last allowed key column
  const int chunks = (int)(cols >> 3);
  float v[kSmMaxChunks][8];
  float m = -INFINITY;
#pragma unroll
  for (int c = 0; c < kSmMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks && ci * 8 <= last) {
      const float4 a = *reinterpret_cast<const float4*>(s + base + (int64_t)ci * 8);
      const float4 b = *reinterpret_cast<const float4*>(s + base + (int64_t)ci * 8 + 4);
      const float t[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        v[c][j] = (ci * 8 + j <= last) ? t[j] * scale : -INFINITY;
        m = fmaxf(m, v[c][j]);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[c][j] = -INFINITY;
    }
  }
  m = block_reduce<true>(m, red);  // finite: column 0 is always allowed
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kSmMaxChunks; ++c)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      v[c][j] = expf(v[c][j] - m);  // exp(-inf) = 0 for masked columns
      sum += v[c][j];
    }
  sum = block_reduce<false>(sum, red);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int c = 0; c < kSmMaxChunks; ++c) {
    const int ci = threadIdx.x + 256 * c;
    if (ci < chunks) {
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = pack2(v[c][2 * j] * inv, v[c][2 * j + 1] * inv);
      *reinterpret_cast<uint4*>(out + base + (int64_t)ci * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// one thread per 4 output elements
__global__ __launch_bounds__(256) void silu_mul_kernel(const float* __restrict__ gu, int64_t rows, int64_t width,
                                                       uint16_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_row = width >> 2;
  if (idx >= rows * per_row) return;
  const int64_t r = idx / per_row, c = (idx - r * per_row) * 4;
  const float4 g = *reinterpret_cast<const float4*>(gu + r * 2 * width + c);
  const float4 u = *reinterpret_cast<const float4*>(gu + r * 2 * width + width + c);
  const float gg[4] = {g.x, g.y, g.z, g.w}, uu[4] = {u.x, u.y, u.z, u.w};
  float o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) o[j] = silu_mul_value(gg[j], uu[j]);
  *reinterpret_cast<uint2*>(out + r * width + c) = make_uint2(pack2(o[0], o[1]), pack2(o[2], o[3]));
}

__global__ __launch_bounds__(256) void residual_add_kernel(const uint16_t* __restrict__ x, const float* __restrict__ y,
                                                           int64_t n4, uint16_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n4) return;
  const uint2 xv = *reinterpret_cast<const uint2*>(x + idx * 4);
  const float4 yv = *reinterpret_cast<const float4*>(y + idx * 4);
  const float a0 = u2f(xv.x << 16) + yv.x, a1 = u2f(xv.x & 0xFFFF0000u) + yv.y;
  const float a2 = u2f(xv.y << 16) + yv.z, a3 = u2f(xv.y & 0xFFFF0000u) + yv.w;
  *reinterpret_cast<uint2*>(out + idx * 4) = make_uint2(pack2(a0, a1), pack2(a2, a3));
}

// one thread per 4 elements of the output row
__global__ __launch_bounds__(256) void merge_heads_kernel(const float* __restrict__ in, int64_t groups,
                                                          int64_t per_group, int64_t seq, int64_t head_dim,
                                                          uint16_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t width = groups * per_group * head_dim, per_row = width >> 2;
  if (idx >= seq * per_row) return;
  const int64_t s = idx / per_row, c = (idx - s * per_row) * 4;
  const int64_t h = c / head_dim, d = c - h * head_dim;
  const int64_t g = h / per_group, j = h - g * per_group;
  const float4 v = *reinterpret_cast<const float4*>(in + ((g * per_group * seq) + j * seq + s) * head_dim + d);
  *reinterpret_cast<uint2*>(out + s * width + c) = make_uint2(pack2(v.x, v.y), pack2(v.z, v.w));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }
int done(const char* what) {
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? AMX_OK : report_hip_error(e, what);
}

}  // namespace

bool rmsnorm_quantize_supported(int64_t group_size, int64_t dim) {
  return (group_size == 16 || group_size == 32 || group_size == 64) && dim > 0 && dim % group_size == 0 &&
         dim <= 256 * 8 * kRmsMaxChunks;
}

hipError_t launch_rmsnorm_quantize(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, const float* y,
                                   uint16_t* sum_out, const float* weight, int64_t rows, int64_t dim, float eps,
                                   uint8_t* codes, uint8_t* scales, hipStream_t s) {
  if (!rmsnorm_quantize_supported(group_size, dim)) return hipErrorInvalidValue;
  const int lanes_log2 = group_size == 16 ? 1 : group_size == 32 ? 2 : 3;
  auto go = [&]<int SK, bool ASYM>() {
    if (y)
      hipLaunchKernelGGL((rmsnorm_quantize_kernel<SK, ASYM, true>), dim3((unsigned)rows), dim3(256), 0, s, x, y, sum_out,
                         weight, dim, eps, lanes_log2, codes, scales);
    else
      hipLaunchKernelGGL((rmsnorm_quantize_kernel<SK, ASYM, false>), dim3((unsigned)rows), dim3(256), 0, s, x, y,
                         sum_out, weight, dim, eps, lanes_log2, codes, scales);
    return hipGetLastError();
  };
  switch (scale_kind) {
    case kScaleE5M2: return asym ? go.template operator()<kScaleE5M2, true>() : go.template operator()<kScaleE5M2, false>();
    case kScaleE4M3: return asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>();
    case kScaleE8M0Floor:
      return asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
    case kScaleE8M0Round:
      return asym ? go.template operator()<kScaleE8M0Round, true>() : go.template operator()<kScaleE8M0Round, false>();
    default: return hipErrorInvalidValue;
  }
}

}  // namespace amx

using namespace amx;

extern "C" {

int amxfp4_rmsnorm(const void* x_bf16, const float* weight, int64_t rows, int64_t dim, float eps, void* out_bf16,
                   void* stream) {
  if (!x_bf16 || !weight || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "rmsnorm: NULL pointer");
  if (rows <= 0 || dim <= 0 || dim % 8 || dim > 256 * 8 * kRmsMaxChunks || rows > 0x7FFFFFFF)
    return report_error(AMX_ERR_INVALID_ARG, "rmsnorm: rows must be positive, dim a positive multiple of 8 up to 16384");
  if (!aligned16(x_bf16) || !aligned16(weight) || !aligned16(out_bf16))
    return report_error(AMX_ERR_INVALID_ARG, "rmsnorm: pointers must be 16-byte aligned");
  hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)rows), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const uint16_t*>(x_bf16), weight, dim, eps, reinterpret_cast<uint16_t*>(out_bf16));
  return done("rmsnorm launch");
}

int amxfp4_split_heads_rope(const float* in, int64_t seq, int64_t ld, int64_t col0, int64_t heads, int64_t head_dim,
                            int32_t rotate, int64_t pos0, double theta, void* out_bf16, void* stream) {
  if (!in || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope: NULL pointer");
  if (seq <= 0 || heads <= 0 || head_dim <= 0 || head_dim % 2 || head_dim > 256 || col0 < 0 ||
      ld < col0 + heads * head_dim || pos0 < 0)
    return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope: bad shape");
  if (rotate && !(theta > 1.0)) return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope: theta must exceed 1");
  const int64_t threads = seq * (head_dim / 2), head_chunks = (heads + kRopeHeads - 1) / kRopeHeads;
  if (threads > (int64_t)0x7FFFFFFF * 256 || head_chunks > 65535)
    return report_error(AMX_ERR_UNSUPPORTED, "split_heads_rope: too large");
  hipLaunchKernelGGL(split_heads_rope_kernel, dim3(blocks_for(threads), (unsigned)head_chunks), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), in, seq, ld, col0, heads, (int)(head_dim / 2),
                     (int)(rotate != 0), pos0, rotate ? log(theta) : 0.0, reinterpret_cast<uint16_t*>(out_bf16));
  return done("split_heads_rope launch");
}

int amxfp4_split_heads_rope_quantize(const amx_format_t* fmt, const float* in, int64_t seq, int64_t ld, int64_t col0,
                                     int64_t heads, int64_t head_dim, int64_t pos0, double theta, uint8_t* codes,
                                     uint8_t* scales, void* stream) {
  if (!fmt || !in || !codes || !scales) return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope_quantize: NULL pointer");
  if (fmt->elem != AMX_ELEM_FP4_E2M1 || fmt->scale < AMX_SCALE_E8M0_FLOOR || fmt->scale > AMX_SCALE_FP8_E4M3 ||
      (fmt->asymmetric != 0 && fmt->asymmetric != 1))
    return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope_quantize: bad format");
  if (fmt->group_size != 32) return report_error(AMX_ERR_UNSUPPORTED, "split_heads_rope_quantize: groups of 32 only");
  if (seq <= 0 || heads <= 0 || head_dim <= 0 || col0 < 0 || ld < col0 + heads * head_dim || pos0 < 0)
    return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope_quantize: bad shape");
  if (head_dim % 64 || head_dim > 256)
    return report_error(AMX_ERR_UNSUPPORTED, "split_heads_rope_quantize: head_dim must be 64, 128, 192 or 256");
  if (!(theta > 1.0)) return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope_quantize: theta must exceed 1");
  if (!aligned16(in) || ld % 4 || col0 % 4 || (reinterpret_cast<uintptr_t>(codes) & 3) || (reinterpret_cast<uintptr_t>(scales) & 1))
    return report_error(AMX_ERR_INVALID_ARG, "split_heads_rope_quantize: in must be 16-byte aligned with ld and col0 multiples "
                        "of 4, codes 4-byte and scales 2-byte aligned");
  const int64_t threads = seq * (head_dim / 16), head_chunks = (heads + kRopeHeads - 1) / kRopeHeads;
  if (threads > (int64_t)0x7FFFFFFF * 256 || head_chunks > 65535)
    return report_error(AMX_ERR_UNSUPPORTED, "split_heads_rope_quantize: too large");
  const dim3 grid(blocks_for(threads), (unsigned)head_chunks);
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  const int half = (int)(head_dim / 2);
  const double lt = log(theta);
  auto go = [&]<int SK, bool ASYM>() {
    hipLaunchKernelGGL((rope_quantize_kernel<SK, ASYM>), grid, dim3(256), 0, hs, in, seq, ld, col0, heads, half, pos0, lt,
                       codes, scales);
  };
  const bool asym = fmt->asymmetric != 0;
  switch (fmt->scale) {
    case AMX_SCALE_FP8_E5M2: asym ? go.template operator()<kScaleE5M2, true>() : go.template operator()<kScaleE5M2, false>(); break;
    case AMX_SCALE_FP8_E4M3: asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>(); break;
    case AMX_SCALE_E8M0_FLOOR:
      asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
      break;
    default: asym ? go.template operator()<kScaleE8M0Round, true>() : go.template operator()<kScaleE8M0Round, false>();
  }
  return done("split_heads_rope_quantize launch");
}

int amxfp4_softmax_causal(const float* scores, int64_t batch, int64_t rows, int64_t cols, float scale, void* out_bf16,
                          void* stream) {
  if (!scores || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "softmax_causal: NULL pointer");
  if (batch <= 0 || rows <= 0 || cols <= 0 || cols % 8 || cols > 256 * 8 * kSmMaxChunks || batch > 65535 ||
      rows > 0x7FFFFFFF)
    return report_error(AMX_ERR_INVALID_ARG, "softmax_causal: cols must be a positive multiple of 8 up to 16384");
  if (!aligned16(scores) || !aligned16(out_bf16))
    return report_error(AMX_ERR_INVALID_ARG, "softmax_causal: pointers must be 16-byte aligned");
  hipLaunchKernelGGL(softmax_causal_kernel, dim3((unsigned)rows, (unsigned)batch), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), scores, rows, cols, scale,
                     reinterpret_cast<uint16_t*>(out_bf16));
  return done("softmax_causal launch");
}

int amxfp4_silu_mul(const float* gate_up, int64_t rows, int64_t width, void* out_bf16, void* stream) {
  if (!gate_up || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "silu_mul: NULL pointer");
  if (rows <= 0 || width <= 0 || width % 4) return report_error(AMX_ERR_INVALID_ARG, "silu_mul: width % 4 != 0");
  if (!aligned16(gate_up) || (reinterpret_cast<uintptr_t>(out_bf16) & 7))
    return report_error(AMX_ERR_INVALID_ARG, "silu_mul: misaligned pointer");
  hipLaunchKernelGGL(silu_mul_kernel, dim3(blocks_for(rows * (width / 4))), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), gate_up, rows, width, reinterpret_cast<uint16_t*>(out_bf16));
  return done("silu_mul launch");
}

int amxfp4_residual_add(const void* x_bf16, const float* y, int64_t n, void* out_bf16, void* stream) {
  if (!x_bf16 || !y || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "residual_add: NULL pointer");
  if (n <= 0 || n % 4) return report_error(AMX_ERR_INVALID_ARG, "residual_add: n must be a positive multiple of 4");
  if (!aligned16(y) || (reinterpret_cast<uintptr_t>(x_bf16) & 7) || (reinterpret_cast<uintptr_t>(out_bf16) & 7))
    return report_error(AMX_ERR_INVALID_ARG, "residual_add: misaligned pointer");
  hipLaunchKernelGGL(residual_add_kernel, dim3(blocks_for(n / 4)), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const uint16_t*>(x_bf16), y, n / 4, reinterpret_cast<uint16_t*>(out_bf16));
  return done("residual_add launch");
}

int amxfp4_merge_heads(const float* in, int64_t groups, int64_t per_group, int64_t seq, int64_t head_dim,
                       void* out_bf16, void* stream) {
  if (!in || !out_bf16) return report_error(AMX_ERR_INVALID_ARG, "merge_heads: NULL pointer");
  if (groups <= 0 || per_group <= 0 || seq <= 0 || head_dim <= 0 || head_dim % 4)
    return report_error(AMX_ERR_INVALID_ARG, "merge_heads: bad shape");
  if (!aligned16(in) || (reinterpret_cast<uintptr_t>(out_bf16) & 7))
    return report_error(AMX_ERR_INVALID_ARG, "merge_heads: misaligned pointer");
  hipLaunchKernelGGL(merge_heads_kernel, dim3(blocks_for(seq * groups * per_group * head_dim / 4)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), in, groups, per_group, seq, head_dim,
                     reinterpret_cast<uint16_t*>(out_bf16));
  return done("merge_heads launch");
}

}  // extern "C"
