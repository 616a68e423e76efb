// Internal launch interface between the C-ABI layer (api.hip) and the kernel files. Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace amx {

// Scale formats (values of amx_scale_t in include/amxfp4.h).
enum : int { kScaleE8M0Floor = 0, kScaleE8M0Round = 1, kScaleE5M2 = 2, kScaleE4M3 = 3 };

// GEMM tiling of the BF16-expanded path: operands are expanded into MFMA-fragment-major BF16 panels whose row count
// is padded to kPanelRows and whose K is padded to kPanelK, so that the GEMM main loop needs no bounds checks.
constexpr int kPanelRows = 256;
constexpr int kPanelK = 128;

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// Group sizes (Sec. 2.1; the code example of Appendix B uses one group per row, written as group size -1). Kernels
// take log2 of the size and find an element's group with a shift; a whole-row group is the shift kWholeRowLog2,
// which sends every element index below 2^31 to group 0.
constexpr int kWholeRowLog2 = 31;
// log2 of a supported group size (16, 32, 64, 128), kWholeRowLog2 for -1, else -1
inline int group_log2(int64_t gs) {
  return gs == 16 ? 4 : gs == 32 ? 5 : gs == 64 ? 6 : gs == 128 ? 7 : gs == -1 ? kWholeRowLog2 : -1;
}
inline bool group_divides(int64_t K, int64_t gs) { return gs == -1 || (gs > 0 && K % gs == 0); }
// groups in a row of K elements
__host__ __device__ inline int64_t groups_per_row(int64_t K, int gs_log2) {
  return gs_log2 == kWholeRowLog2 ? 1 : K >> gs_log2;
}

// api.hip: status reporting shared by all entry points (thread-local message behind amxfp4_last_error)
int report_error(int code, const char* msg);
int report_hip_error(hipError_t e, const char* what);

// cast.hip (group_size: 16, 32, 64 or 128, dividing K, or -1 for whole rows, contiguous rows only; tensor_pair: device {S_t, 1 / S_t} of a tensor-wise scale,
// or null for none; batch operands batch_stride elements apart, their outputs packed one after the other)
hipError_t launch_quantize_contig(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, int64_t rows,
                                  int64_t K, int64_t row_stride, int64_t batch, int64_t batch_stride,
                                  const float* tensor_pair, uint8_t* codes, uint8_t* scales, hipStream_t s);
hipError_t launch_quantize_strided(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, int64_t rows,
                                   int64_t K, int64_t k_stride, int64_t batch, int64_t batch_stride,
                                   const float* tensor_pair, uint8_t* codes, uint8_t* scales, hipStream_t s);
hipError_t launch_dequantize(int scale_kind, bool asym, int64_t group_size, const uint8_t* codes,
                             const uint8_t* scales, int64_t rows, int64_t K, const float* tensor_pair, void* out,
                             int out_dtype, hipStream_t s);
hipError_t launch_tensor_scale(const uint16_t* x, int64_t rows, int64_t K, int64_t row_stride, float* pair,
                               hipStream_t s);

// Optional event pair recorded around the matrix-multiply kernel of one GEMM call (measurement aid).
struct KernelTimer {
  hipEvent_t start = nullptr, stop = nullptr;
};

// gemm_bf16.hip (glu: the gated-activation epilogue; C is then the BF16 output [M][ldc] of N / 2 columns;
// tile: 0 = chosen by a cost model over the shape, 1 = 256 x 256, 2 = 256 x 128, 3 = 64 x 256)
size_t bf16_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch);
hipError_t launch_gemm_bf16_path(int scale_kind, bool asym, int64_t group_size, int64_t M, int64_t N, int64_t K,
                                 const uint8_t* A_codes, const uint8_t* A_scales, const uint8_t* B_codes,
                                 const uint8_t* B_scales, const float* A_tensor_pair, const float* B_tensor_pair,
                                 float* C, int64_t ldc, int64_t batch, void* workspace, int tile, hipStream_t s,
                                 const KernelTimer& timer, bool glu = false, const void* B_panel = nullptr);
// B's panel alone, expanded once for weights that stay (bf16_panel_bytes(N, K) bytes); passed as B_panel above, the
// call then expands only A and its workspace is bf16_panel_bytes(M, K) per batch entry.
size_t bf16_panel_bytes(int64_t rows, int64_t K);
hipError_t launch_expand_b_panel(int scale_kind, bool asym, int64_t group_size, int64_t N, int64_t K,
                                 const uint8_t* B_codes, const uint8_t* B_scales, void* panel, hipStream_t s);

// BF16 fragment-major panel [batch][Rp / 32][Kp / 16][64 lanes][8] of a quantized operand (rows >= R and columns >= K
// zero; Rp % 32 == 0, Kp % 64 == 0). permute: the key order of the fused attention kernel's V operand (gemm_bf16.hip).
hipError_t launch_expand_bf16(int scale_kind, bool asym, int64_t group_size, const uint8_t* codes,
                              const uint8_t* scales, int64_t R, int64_t K, int64_t Rp, int64_t Kp, int64_t batch,
                              bool permute, uint16_t* panel, hipStream_t s);
// (a permuted panel of an FP8-E5M2 operand is FP16 biased by 2^-3 instead of BF16: what the attention kernel's second
// product takes for that scale format)

// gemm_skinny.hip: M <= 256, K a multiple of 256, groups of 32: B dequantized in registers straight from its codes
// (workspace: the BF16 panel of A and, with several outer K slices, the partial tiles; forced_slices: 0 = the number
// of outer K slices comes from a cost model, n > 0 = n of them, at most K / 256)
bool skinny_path_supported(int64_t M, int64_t N, int64_t K, int64_t batch);
size_t skinny_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int forced_slices);
hipError_t launch_gemm_skinny_path(int scale_kind, bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                   const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                   int64_t ldc, int64_t batch, void* workspace, int forced_slices, hipStream_t s,
                                   const KernelTimer& timer);

// attention.hip: fused quantized attention, head dimension 128 or 64, groups of 32 (workspace: the three BF16 panels).
// merged_bf16: out is BF16 [Sq][Hq * head_dim] (token-major) instead of FP32 [Hq][Sq][head_dim]
size_t attention_workspace_bytes(int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk, int64_t head_dim);
hipError_t launch_attention_fused(int scale_kind, bool asym, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk,
                                  int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales,
                                  const uint8_t* K_codes, const uint8_t* K_scales, const uint8_t* V_codes,
                                  const uint8_t* V_scales, float scale, int causal, float* out, bool merged_bf16,
                                  void* workspace, hipStream_t s, const KernelTimer& timer);

// attention_decode.hip: the same attention for few queries ((Hq / Hkv) * Sq <= 32) against many keys, K and V read as
// packed codes, the key tiles cut into key_splits ranges (workspace: the ranges' partial results)
bool attention_decode_supported(int64_t Hq, int64_t Hkv, int64_t Sq, int64_t head_dim);
size_t attention_decode_workspace_bytes(int64_t Hkv, int64_t head_dim, int64_t key_splits);
hipError_t launch_attention_decode(int scale_kind, bool asym, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk,
                                   int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales,
                                   const uint8_t* K_codes, const uint8_t* K_scales, const uint8_t* V_codes,
                                   const uint8_t* V_scales, float scale, int causal, int key_splits, float* out,
                                   void* workspace, hipStream_t s);

// layer_ops.hip: RMS normalisation (after an optional residual addition y, whose BF16 sum goes to sum_out) with the
// cast of the normalised row fused in; groups of 16, 32 or 64 dividing dim <= 16384
bool rmsnorm_quantize_supported(int64_t group_size, int64_t dim);
hipError_t launch_rmsnorm_quantize(int scale_kind, bool asym, int64_t group_size, const uint16_t* x, const float* y,
                                   uint16_t* sum_out, const float* weight, int64_t rows, int64_t dim, float eps,
                                   uint8_t* codes, uint8_t* scales, hipStream_t s);

// The A panel of the few-rows kernel: 32-long groups, FP16 biased by 2^-3 for FP8-E5M2 scales and BF16 otherwise, the
// k order within every block of 256 rearranged so that a lane half's 16 k-steps come from one half of the block
// (gemm_bf16.hip, HALF_LINE). K % 256 == 0.
hipError_t launch_expand_half_line(int scale_kind, bool asym, const uint8_t* codes, const uint8_t* scales, int64_t R,
                                   int64_t K, int64_t Rp, int64_t batch, uint16_t* panel, hipStream_t s);
// FP16 fragment-major panel (values biased by 2^-3) of an operand with FP8-E5M2 scales; layout as the BF16 panels
hipError_t launch_expand_f16_e5m2(bool asym, const uint8_t* codes, const uint8_t* scales, int64_t R, int64_t K,
                                  int64_t Rp, int64_t Kp, int64_t batch, uint16_t* panel, hipStream_t s);

// gemm_fp4.hip: power-of-two scales on the block-scaled FP4 MFMA (workspace: the scale bytes re-laid in the order the
// waves fetch them). glu here and below: as for the BF16 path
bool fp4_path_supported(int64_t M, int64_t N, int64_t K);
size_t fp4_path_workspace_bytes(bool asym, int64_t M, int64_t N, int64_t K, int64_t batch);
hipError_t launch_gemm_fp4_path(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                int64_t ldc, int64_t batch, void* workspace, hipStream_t s, const KernelTimer& timer,
                                bool glu = false);

// gemm_fp8m.hip: asymmetric power-of-two scales merged per group into E5M2 elements + one anchor scale, block-scaled
// FP8 MFMA (workspace: the merged panels)
size_t fp8m_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch);
hipError_t launch_gemm_fp8m_path(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                 const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc, int64_t batch,
                                 void* workspace, hipStream_t s, const KernelTimer& timer, bool glu = false);

// gemm_fp6m.hip: asymmetric power-of-two scales merged per group into FP6 (E3M2) elements + one anchor scale, block-
// scaled MFMA at the FP4 rate; group positions whose scales lie too far apart for one FP6 operand are written twice
// along K, split by sign (workspace: merged panels sized for the worst case, anchors, the split plan)
bool fp6m_path_supported(int64_t M, int64_t N, int64_t K);
size_t fp6m_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch);
hipError_t launch_gemm_fp6m_path(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                 const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc, int64_t batch,
                                 void* workspace, hipStream_t s, const KernelTimer& timer, bool glu = false);
// the same on prepared weights: B's panel (its own blocks), anchors and plan written once (fp6m_prepared_bytes(N, K)
// bytes); the call then flags and merges only A (workspace: A's panel and anchors, B's anchors in the call's K order,
// the plan with the table of B blocks)
size_t fp6m_prepared_bytes(int64_t N, int64_t K);
size_t fp6m_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K);
hipError_t launch_fp6m_prepare_b(int64_t N, int64_t K, const uint8_t* B_codes, const uint8_t* B_scales, void* prepared,
                                 hipStream_t s);
hipError_t launch_gemm_fp6m_prepared(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                     const void* prepared, float* C, int64_t ldc, void* workspace, hipStream_t s,
                                     const KernelTimer& timer, bool glu = false);

// gemm_e5m2.hip: FP8-E5M2 scales, dequantization fused into the FP16-MFMA kernel (no workspace)
bool e5m2_fused_supported(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemm_e5m2_fused(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                  const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                  int64_t ldc, int64_t batch, hipStream_t s, const KernelTimer& timer);

// FP8-E5M2 scales, A from an FP16 panel in the workspace, B dequantized inside the kernel (workspace: the A panel only)
bool e5m2_hybrid_supported(int64_t M, int64_t N, int64_t K);
size_t e5m2_hybrid_workspace_bytes(int64_t M, int64_t K, int64_t batch);
hipError_t launch_gemm_e5m2_hybrid(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                   const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                   int64_t ldc, int64_t batch, void* workspace, hipStream_t s,
                                   const KernelTimer& timer);

}  // namespace amx
