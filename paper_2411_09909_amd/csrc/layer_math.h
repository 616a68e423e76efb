// Scalar arithmetic shared by the decoder-layer operators (layer_ops.hip) and by the GEMM epilogue that applies one of
// them in registers (gemm_bf16.hip): the two must give the same bits.
#pragma once
#include "device_formats.h"

namespace amx {

// FP32 -> BF16 bit pattern, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = f2u(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return bf16_rne(a) | (bf16_rne(b) << 16); }

// silu(gate) * up in FP32, silu(g) = g / (1 + exp(-g)), with the hardware's exp2 and reciprocal (about an ulp of FP32
// each; the result is rounded to BF16 by every caller, 16 bits coarser). The library's expf and division cost the
// gated GEMM epilogue, which evaluates this 128 times per lane and tile with nothing to hide it behind, 0.08-0.18 ms of
// a 28672-wide gate / up product. A gate below about -88 gives exp = inf, 1 / inf = 0 and the result -0 * up, the limit.
__device__ __forceinline__ float silu_mul_value(float gate, float up) {
  const float e = __builtin_amdgcn_exp2f(gate * -1.4426950408889634f);
  return gate * __builtin_amdgcn_rcpf(1.0f + e) * up;
}

}  // namespace amx
