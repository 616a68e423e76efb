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

// silu(gate) * up in FP32, silu(g) = g / (1 + exp(-g))
__device__ __forceinline__ float silu_mul_value(float gate, float up) { return gate / (1.0f + expf(-gate)) * up; }

}  // namespace amx
