/*
 * libamxfp4 — glue operators of the decoder-layer workload.
 *
 * The paper quantizes every matrix multiplication of a transformer decoder layer (Sec. 5.1, evaluation setup: the
 * linear projections and the two attention products Q.K^T and P.V) and leaves the operators between them in BF16.
 * These entry points are those operators for a LLaMA-style layer, so that a whole layer can run through the
 * quantized GEMM of amxfp4.h without leaving the device: they take the FP32 outputs of amxfp4_gemm and produce the
 * BF16 operands of the next amxfp4_quantize. None of them is part of the paper's method.
 *
 * Conventions as in amxfp4.h: every data pointer is a DEVICE pointer owned by the caller, nothing is allocated or
 * retained, calls are asynchronous on `stream` (hipStream_t as void*), arguments are validated on the host before
 * any launch, the return value is an amx_status_t and the message is available from amxfp4_last_error().
 * "bf16" buffers hold BF16 bit patterns (uint16); FP32 -> BF16 conversions round to nearest even.
 */
#ifndef AMXFP4_LAYER_H
#define AMXFP4_LAYER_H

#include <stddef.h>
#include <stdint.h>

#include "amxfp4.h" /* amx_format_t, status codes */

#ifdef __cplusplus
extern "C" {
#endif

/*
 * RMS normalisation of each row: out[r, c] = bf16( x[r, c] * rsqrt(mean_c(x[r, :]^2) + eps) * weight[c] ), all
 * arithmetic in FP32. x, out: [rows, dim] BF16, contiguous; weight: [dim] FP32. dim must be a multiple of 8 and at
 * most 16384.
 */
int amxfp4_rmsnorm(const void* x_bf16, const float* weight, int64_t rows, int64_t dim, float eps, void* out_bf16,
                   void* stream);

/*
 * Splits a token-major FP32 projection output into heads and (optionally) applies rotary position embedding.
 * in: [seq, ld] FP32; head h occupies columns col0 + h * head_dim .. + head_dim - 1 of every row.
 * out: [heads, seq, head_dim] BF16 (head-major, each head a contiguous [seq, head_dim] matrix).
 * rotate != 0: the pair (i, i + head_dim / 2), i < head_dim / 2, of the token at position p = pos0 + row is rotated
 * by the angle p * theta^(-2 i / head_dim) ("rotate-half" convention: out_i = x_i cos - x_{i+d/2} sin,
 * out_{i+d/2} = x_{i+d/2} cos + x_i sin); the angle and its sine / cosine are evaluated in FP64.
 * rotate == 0: plain conversion and re-layout (values). head_dim must be even and at most 256.
 */
int amxfp4_split_heads_rope(const float* in, int64_t seq, int64_t ld, int64_t col0, int64_t heads, int64_t head_dim,
                            int32_t rotate, int64_t pos0, double theta, void* out_bf16, void* stream);

/*
 * amxfp4_split_heads_rope with rotate != 0 followed by amxfp4_quantize of every head along head_dim (Appendix B
 * Algorithm 1 / Sec. 4.2 Eq. 1; Sec. 5.1 quantizes the operands of Q.K^T), in one pass: the rotated BF16 heads are
 * never written. codes [heads][seq][head_dim / 2] and scales [heads][seq][head_dim / 32] (x 2 when asymmetric) come out
 * bit for bit as from the two separate calls: the Q and K operands of amxfp4_attention.
 *   fmt        group_size 32 (AMX_ERR_UNSUPPORTED otherwise); head_dim 64, 128, 192 or 256
 *   in         [seq][ld] FP32, 16-byte aligned, ld and col0 multiples of 4; other arguments as amxfp4_split_heads_rope
 *   codes      device out, 4-byte aligned; scales device out, 2-byte aligned
 */
int amxfp4_split_heads_rope_quantize(const amx_format_t* fmt, const float* in, int64_t seq, int64_t ld, int64_t col0,
                                     int64_t heads, int64_t head_dim, int64_t pos0, double theta, uint8_t* codes,
                                     uint8_t* scales, void* stream);

/*
 * Causal softmax of attention scores. scores: [batch, rows, cols] FP32, contiguous; row r of every batch entry
 * belongs to the query at position r % cols (several query heads that share one key head may be stacked along the
 * rows); it attends to key columns c <= r % cols. out[b, r, c] = bf16( exp(scale * (s[c] - max)) / sum ) over the
 * allowed columns and exactly 0 elsewhere; FP32 arithmetic. cols at most 16384 and a multiple of 8.
 */
int amxfp4_softmax_causal(const float* scores, int64_t batch, int64_t rows, int64_t cols, float scale, void* out_bf16,
                          void* stream);

/*
 * Gated activation of a fused gate / up projection: in [rows, 2 * width] FP32 with the gate in columns [0, width) and
 * the up projection in [width, 2 * width); out[r, c] = bf16( silu(gate) * up ), silu(g) = g / (1 + exp(-g)), FP32.
 * width must be a multiple of 4.
 */
int amxfp4_silu_mul(const float* gate_up, int64_t rows, int64_t width, void* out_bf16, void* stream);

/*
 * The fused gate / up projection with the gated activation applied before anything is written: out[r, c] =
 * bf16( silu(g) * u ) with (g | u) = the quantized product A . B^T of amxfp4_gemm (Sec. 4.3) and the arithmetic of
 * amxfp4_silu_mul, bit for bit; the FP32 product never goes to memory.
 *   A                  [M][K] quantized activations (codes, scales as for amxfp4_gemm).
 *   B                  [2 * width][K] quantized weights with the rows of the gate and of the up projection INTERLEAVED
 *                      in blocks of 32: rows 64 t .. 64 t + 31 are gate rows 32 t .. 32 t + 31, rows 64 t + 32 ..
 *                      64 t + 63 the up rows of the same indices. width % 32 == 0.
 *   out_bf16           device out, [M][ld_out] BF16 bit patterns, ld_out >= width.
 *   workspace          at least amxfp4_gemm_silu_mul_workspace_bytes() bytes, 256-byte aligned; may be NULL when
 *                      that is 0. The product runs on the tiled kernel of the format (block-scaled matrix
 *                      instructions for power-of-two scales of 32-groups, exact BF16 operands otherwise), whatever M.
 * Status codes as amxfp4_gemm.
 */
size_t amxfp4_gemm_silu_mul_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K);
int amxfp4_gemm_silu_mul(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K, const uint8_t* A_codes,
                         const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, void* out_bf16,
                         int64_t ld_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * amxfp4_gemm_silu_mul on prepared weights: `prepared` is what amxfp4_prepare_weights (include/amxfp4.h) wrote for the
 * INTERLEAVED weight matrix B [2 * width][K]; the call then expands only A. Same result, bit for bit. For formats with
 * nothing to prepare (amxfp4_weights_prepared_bytes() == 0) `prepared` is ignored and the call is amxfp4_gemm_silu_mul.
 * workspace: at least amxfp4_gemm_silu_mul_prepared_workspace_bytes() bytes.
 */
size_t amxfp4_gemm_silu_mul_prepared_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K);
int amxfp4_gemm_silu_mul_prepared(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K, const uint8_t* A_codes,
                                  const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales,
                                  const void* prepared, size_t prepared_bytes, void* out_bf16, int64_t ld_out,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * amxfp4_rmsnorm followed by amxfp4_quantize of its result (Appendix B Algorithm 1 / Sec. 4.2 Eq. 1, as amxfp4_quantize
 * along the row), in one pass: the normalised BF16 row is cast in registers and never written. Optionally with the
 * residual addition of amxfp4_residual_add in front: y != NULL adds the FP32 row y to x first, writes the BF16 sum to
 * sum_out_bf16 (the residual stream a later addition needs) and normalises that sum. codes [rows][dim / 2] and scales
 * (layout of amxfp4_quantize) come out bit for bit as from the separate calls.
 *   fmt        group_size 16, 32 or 64 dividing dim (AMX_ERR_UNSUPPORTED otherwise); dim <= 16384
 *   x_bf16     [rows][dim] BF16, contiguous; y [rows][dim] FP32 or NULL; sum_out_bf16 [rows][dim] BF16, non-NULL
 *              exactly when y is (it may be x itself: every element is read before it is written, by the same lane)
 *   weight     [dim] FP32. x, y, sum_out, weight, codes: 16-byte aligned; scales: 4-byte aligned.
 */
int amxfp4_rmsnorm_quantize(const amx_format_t* fmt, const void* x_bf16, const float* y, void* sum_out_bf16,
                            const float* weight, int64_t rows, int64_t dim, float eps, uint8_t* codes, uint8_t* scales,
                            void* stream);

/* out = bf16( float(x) + y ): x, out [n] BF16, y [n] FP32 (residual connection after a projection). n % 4 == 0. */
int amxfp4_residual_add(const void* x_bf16, const float* y, int64_t n, void* out_bf16, void* stream);

/*
 * Inverse of the head split for the attention output: in [groups, per_group * seq, head_dim] FP32, where row
 * j * seq + s of group g is head g * per_group + j at token s; out [seq, groups * per_group * head_dim] BF16
 * (token-major, head h in columns h * head_dim ..). head_dim % 4 == 0.
 */
int amxfp4_merge_heads(const float* in, int64_t groups, int64_t per_group, int64_t seq, int64_t head_dim,
                       void* out_bf16, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AMXFP4_LAYER_H */
