// Measurement aids (not part of the method): what this machine actually sustains on the two resources the hot path is
// bounded by, to be printed beside the datasheet peaks.
//   - a register-resident MFMA loop: 16 independent accumulator tiles per wave, operands loaded once, no memory
//     traffic inside the loop. Its rate depends on the operand DATA (the chip lowers its clock under load, and more
//     so for operands with many toggling bits), so the caller supplies the operand bits (zeros, or a slice of a real
//     quantized / expanded operand);
//   - a plain streaming copy (128-bit loads and stores, grid-stride).
#include "../../include/amxfp4.h"
#include "gemm_common.h"
#include "kernels.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPeakTiles = 16;     // independent accumulators per wave
constexpr int kPeakBlocks = 512;   // two rounds of one 4-wave workgroup per CU (the accumulators fill the registers)

// KIND 0: v_mfma_f32_32x32x16_bf16; 1: block-scaled 32x32x64 with FP8 (E5M2) operands; 2: the same with FP4 operands;
// 3: v_mfma_f32_32x32x16_f16; 4: the block-scaled instruction with FP6 (E3M2) operands.
// operand: 256 lanes x 2 (A, B) x 32 bytes. sink: kPeakBlocks * 256 floats (keeps the loop alive).
template <int KIND>
__global__ __launch_bounds__(256) void peak_mfma_kernel(const uint8_t* __restrict__ operand, float* __restrict__ sink,
                                                        int iterations) {
  const u32x4* src = reinterpret_cast<const u32x4*>(operand) + threadIdx.x * 4;
  const u32x4 a0 = src[0], a1 = src[1], b0 = src[2], b1 = src[3];
  f32x16 acc[kPeakTiles];
#pragma unroll
  for (int i = 0; i < kPeakTiles; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  if constexpr (KIND == 0) {
    const bf16x8 a = __builtin_bit_cast(bf16x8, a0), b = __builtin_bit_cast(bf16x8, b0);
    for (int it = 0; it < iterations; ++it)
#pragma unroll
      for (int i = 0; i < kPeakTiles; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  } else if constexpr (KIND == 3) {
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    const f16x8 a = __builtin_bit_cast(f16x8, a0), b = __builtin_bit_cast(f16x8, b0);
    for (int it = 0; it < iterations; ++it)
#pragma unroll
      for (int i = 0; i < kPeakTiles; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
  } else {
    // FP4 operands occupy the first four registers of the eight, FP6 the first six; unit block scales (E8M0 byte 127)
    const i32x8 a = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
    const i32x8 b = {(int)b0[0], (int)b0[1], (int)b0[2], (int)b0[3], (int)b1[0], (int)b1[1], (int)b1[2], (int)b1[3]};
    const int unit = 0x7F7F7F7F;
    for (int it = 0; it < iterations; ++it)
#pragma unroll
      for (int i = 0; i < kPeakTiles; ++i) {
        if constexpr (KIND == 1)
          acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 1, 1, 0, unit, 0, unit);
        else if constexpr (KIND == 4)
          acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 3, 3, 0, unit, 0, unit);
        else
          acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4, 4, 0, unit, 0, unit);
      }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kPeakTiles; ++i) s += acc[i][0] + acc[i][15];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void peak_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                        int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace amx

extern "C" {

int amxfp4_peak_mfma(int32_t mfma, const void* operand, int32_t iterations, float* sink, double* flops,
                     void* stream) {
  using namespace amx;
  if (mfma < 0 || mfma > 4)
    return report_error(AMX_ERR_INVALID_ARG, "mfma must be 0 (bf16), 1 (fp8), 2 (fp4), 3 (f16) or 4 (fp6)");
  if (!operand || !sink || !flops) return report_error(AMX_ERR_INVALID_ARG, "NULL pointer");
  if (iterations <= 0 || iterations > (1 << 22)) return report_error(AMX_ERR_INVALID_ARG, "iterations out of range");
  if (reinterpret_cast<uintptr_t>(operand) & 15) return report_error(AMX_ERR_INVALID_ARG, "operand must be 16-byte aligned");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const uint8_t* op = reinterpret_cast<const uint8_t*>(operand);
  if (mfma == 0)
    hipLaunchKernelGGL(peak_mfma_kernel<0>, dim3(kPeakBlocks), dim3(256), 0, s, op, sink, iterations);
  else if (mfma == 1)
    hipLaunchKernelGGL(peak_mfma_kernel<1>, dim3(kPeakBlocks), dim3(256), 0, s, op, sink, iterations);
  else if (mfma == 2)
    hipLaunchKernelGGL(peak_mfma_kernel<2>, dim3(kPeakBlocks), dim3(256), 0, s, op, sink, iterations);
  else if (mfma == 3)
    hipLaunchKernelGGL(peak_mfma_kernel<3>, dim3(kPeakBlocks), dim3(256), 0, s, op, sink, iterations);
  else
    hipLaunchKernelGGL(peak_mfma_kernel<4>, dim3(kPeakBlocks), dim3(256), 0, s, op, sink, iterations);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return report_hip_error(e, "peak probe launch");
  *flops = 2.0 * 32 * 32 * (mfma == 0 || mfma == 3 ? 16 : 64) * kPeakTiles * (double)iterations * 4 * kPeakBlocks;
  return AMX_OK;
}

int amxfp4_peak_copy(const void* src, void* dst, size_t bytes, void* stream) {
  using namespace amx;
  if (!src || !dst || bytes == 0 || bytes % 16 != 0) return report_error(AMX_ERR_INVALID_ARG, "need non-NULL buffers and a multiple of 16 bytes");
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)
    return report_error(AMX_ERR_INVALID_ARG, "buffers must be 16-byte aligned");
  const int64_t n16 = (int64_t)(bytes / 16);
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;  // 16 workgroups per CU, grid-stride beyond
  hipLaunchKernelGGL(peak_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), n16);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? AMX_OK : report_hip_error(e, "copy probe launch");
}

}  // extern "C"
