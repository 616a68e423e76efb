/*
 * amxfp4.h — C ABI of libamxfp4: direct-cast BF16 -> AMXFP4 / MXFP4 group quantization and the fully
 * quantized matrix multiplication that consumes the quantized operands, for AMD MI355X (gfx950).
 *
 * Formats (paper Sec. 2.1, Sec. 4.2 Eq. 1, Sec. 4.3, Appendix B Algorithm 1 and the table of MX-compliant formats):
 *   element   FP4 E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit; magnitudes {0, .5, 1, 1.5, 2, 3, 4, 6}.
 *   group     `group_size` consecutive elements along the contraction axis K share the scale(s): 32 in MX and in
 *             the paper's format; 16, 64 and 128 are the other points of its group-size study (Sec. 5.3, Table 5);
 *             -1 makes each row one group, as the code example of Appendix B does (there K / group_size reads 1).
 *             The contiguous cast, the dequantization and the amxfp4_gemm* calls take -1; every other call
 *             returns AMX_ERR_UNSUPPORTED for it.
 *   MXFP4     one scale S per group;            x_hat = (-1)^s * elem * S
 *   AMXFP4    two scales (S_p, S_n) per group;  x_hat = (-1)^s * elem * (s == 0 ? S_p : S_n)         (Eq. 1)
 *   scale     8 bits: E8M0 power of two (Algorithm 1, exponent floored), or FP8 E5M2 (Sec. 4.2 "FP8";
 *             this is the format the paper calls AMXFP4 when asymmetric and "MXFP4" in its result tables when
 *             symmetric), or FP8 E4M3 (Sec. 4.2: the FP8 scale with one more mantissa bit and less range).
 *   product   every elementwise product in a dot product carries the scale pair picked by the signs of its
 *             two factors (Sec. 4.3); accumulation is FP32 on the GPU.
 *
 * Quantization rule (Algorithm 1; Sec. 4.2; Appendix B worked example), per group and per sign class c in {p, n}:
 *   amax_p = largest positive element (0 if none), amax_n = largest |negative element| (0 if none);
 *   symmetric formats use amax = max(amax_p, amax_n) for both classes.
 *   E5M2      S_c = round-to-nearest-even onto the non-negative E5M2 values of the real quotient amax_c / 6,
 *             saturating at 57344, subnormals kept;
 *   E4M3      the same onto the non-negative E4M3 values (OCP FP8: bias 7, largest finite value 448);
 *   E8M0      S_c = 2^(floor(log2 amax_c) - 2)  (S_c byte 0 when amax_c == 0);
 *   element   magnitude = round-to-nearest (ties to the even code) of min(|x| / S_c, 6) onto the E2M1 grid,
 *             0 when S_c == 0; sign bit copied from the input's IEEE sign bit.
 *
 * Storage (the paper gives none; this layout is this library's):
 *   codes     row-major [rows][K/2] bytes; byte b holds element 2b in bits 3:0 and element 2b+1 in bits 7:4;
 *             nibble = s e1 e0 m.
 *   scales    asymmetric: row-major [rows][K/group_size][2] bytes = (S_p, S_n); symmetric: [rows][K/group_size].
 *             E5M2 byte = 0eeeeemm, bias 15, subnormals m * 2^-16.  E4M3 byte = 0eeeemmm, bias 7, subnormals
 *             m * 2^-9.  E8M0 byte = exponent + 127.
 *
 * Conventions for every entry point below:
 *   - all data pointers are DEVICE pointers owned by the caller unless stated otherwise; the library never
 *     frees or retains them; `fmt` is a HOST pointer read during the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Work is enqueued on it and the
 *     call returns without synchronising.
 *   - arguments are validated on the host before anything is launched; on a non-zero return no output byte has
 *     been written. Inputs must be finite BF16 (NaN/Inf give unspecified codes but never an out-of-bounds access).
 *   - returns AMX_OK or a negative amx_status_t; amxfp4_last_error() gives a thread-local message.
 *   - no process-wide state: nothing is read from the environment and no call changes what a later call does. The
 *     only state is per host thread (the message of amxfp4_last_error and the event pair armed by
 *     amxfp4_profile_next_gemm), so the entry points may be called from several threads at once.
 *   - size limits (AMX_ERR_INVALID_ARG beyond them): K <= 2^20 for every operand; rows of a cast <= 2^31 - 1
 *     (16 776 960 when the groups run down a strided axis); M and N of a GEMM <= 2^21 - 256, ldc <= 2^22; batch <= 65535.
 *     Zero-sized operands are invalid arguments, not no-ops.
 */
#ifndef AMXFP4_H
#define AMXFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AMX_OK = 0,
  AMX_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, K not a multiple of the group, bad enum, misalignment */
  AMX_ERR_UNSUPPORTED = -2, /* a legal format this GPU library, or this call, does not implement (e.g. group_size 8) */
  AMX_ERR_WORKSPACE = -3,   /* workspace missing or smaller than amxfp4_gemm_workspace_bytes() */
  AMX_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed */
} amx_status_t;

typedef enum {
  AMX_ELEM_FP4_E2M1 = 0 /* Sec. 2.1; table of MX-compliant formats */
} amx_elem_t;

typedef enum {
  AMX_SCALE_E8M0_FLOOR = 0, /* OCP MX power-of-two scale, exponent floored (Appendix B, Algorithm 1) */
  AMX_SCALE_E8M0_ROUND = 1, /* power-of-two scale with the exponent rounded instead of floored (Appendix B, "Floor vs. Round") */
  AMX_SCALE_FP8_E5M2 = 2,   /* FP8 scale with a 5-bit exponent, the paper's choice (Sec. 4.2 "FP8") */
  AMX_SCALE_FP8_E4M3 = 3    /* FP8 scale with a 4-bit exponent and 3 mantissa bits (Sec. 4.2; the group scale of NVFP4 in Sec. 5.3) */
} amx_scale_t;

typedef struct {
  int32_t group_size; /* elements per group along K: 16, 32 (Sec. 2.1), 64 or 128, dividing K; -1: the whole row */
  int32_t elem;       /* amx_elem_t */
  int32_t scale;      /* amx_scale_t */
  int32_t asymmetric; /* 1 = AMXFP4: sign-dependent scale pair (Eq. 1); 0 = MXFP4: one scale per group */
} amx_format_t;

/* Human-readable description of the last non-zero status returned on this thread (never NULL). */
const char* amxfp4_last_error(void);

/* Size in bytes of the packed code array for a [rows][K] operand: rows*K/2. 0 on invalid arguments. */
size_t amxfp4_codes_bytes(const amx_format_t* fmt, int64_t rows, int64_t K);
/* Size in bytes of the scale array: rows*(K/group_size)*(asymmetric ? 2 : 1), one group per row for group_size -1.
 * 0 on invalid arguments. */
size_t amxfp4_scales_bytes(const amx_format_t* fmt, int64_t rows, int64_t K);
/* Device scratch amxfp4_gemm needs for `batch` problems of shape M x N x K in this format (may be 0): operand panels
 * for the formats multiplied as 16-bit, FP6 or FP8 values, the re-laid scale bytes for the FP4 kernels. */
size_t amxfp4_gemm_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, int64_t batch);

/*
 * Direct-cast quantization (Algorithm 1 generalised by Sec. 4.2 / Eq. 1; rule restated at the top of this file).
 *   x_bf16      device, BF16 bit patterns; element (r, k) is x_bf16[r*row_stride + k*k_stride] (strides in elements).
 *               k_stride == 1 is the contiguous case (16-byte aligned base, row_stride % 8 == 0);
 *               row_stride == 1 with k_stride >= rows quantizes along a strided axis (groups run down a column,
 *               e.g. V in softmax(P).V, grouped along the key sequence).
 *   rows, K     operand shape; K % group_size == 0 and K % 32 == 0. Whole-row groups: contiguous case only.
 *   codes       device out, amxfp4_codes_bytes() bytes, 16-byte aligned.
 *   scales      device out, amxfp4_scales_bytes() bytes, 4-byte aligned.
 */
int amxfp4_quantize(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                    int64_t k_stride, uint8_t* codes, uint8_t* scales, void* stream);

/*
 * The same cast over `batch` operands of one shape in one launch (the heads of an attention layer, Sec. 5.1: Q, K
 * along the head dimension, V down the keys): operand b starts batch_stride elements after operand b - 1; codes and
 * scales are written packed, [batch][rows][K/2] and [batch][rows][K/group_size]([2]). 1 <= batch <= 65535;
 * batch_stride >= 0 and, for the contiguous case, a multiple of 8. Everything else as amxfp4_quantize.
 */
int amxfp4_quantize_batched(const amx_format_t* fmt, const void* x_bf16, int64_t batch, int64_t batch_stride,
                            int64_t rows, int64_t K, int64_t row_stride, int64_t k_stride, uint8_t* codes,
                            uint8_t* scales, void* stream);

/*
 * Dequantization x_hat = (-1)^s * elem * S_class (Eq. 1), exact in both output types.
 *   out         device out, row-major [rows][K]; out_dtype 0 = float32, 1 = BF16 bit patterns.
 */
int amxfp4_dequantize(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                      void* out, int32_t out_dtype, void* stream);

/*
 * Fully quantized GEMM (Sec. 4.3): C[b][i][j] = sum_k A_hat[b][i][k] * B_hat[b][j][k], with A_hat, B_hat the
 * dequantized operands of Eq. 1, so that each product is scaled by the pair of scales its two signs select.
 * FP32 accumulation, FP32 output.
 *   A_codes/A_scales   [batch][M][K] operand, K contiguous, layouts as above (both operands use `fmt`).
 *   B_codes/B_scales   [batch][N][K] operand, K contiguous (C = A . B^T).
 *   C                  device out, [batch][M][ldc] floats, ldc >= N; columns >= N are not touched.
 *   batch              number of independent back-to-back problems (attention heads), >= 1.
 *   Groups of 32 with power-of-two scales run on the block-scaled FP4 / FP8 matrix instructions; FP8 scales and the
 *   other group sizes are multiplied as exact BF16 operands (element * scale has at most 6 significant bits). With
 *   M <= 256 (M <= 768 for batch == 1 and N * K >= 2^27), groups of 32 and K a multiple of 256, B is read as packed
 *   codes and dequantized in registers to exact 16-bit floats (the weights-bound case of a few tokens against a
 *   weight matrix); results do not depend on the kernel beyond the FP32 summation order.
 *   workspace          device scratch of at least amxfp4_gemm_workspace_bytes() bytes, 256-byte aligned;
 *                      contents are undefined afterwards. May be NULL when the required size is 0.
 */
int amxfp4_gemm(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                int64_t batch, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Static weights. amxfp4_gemm re-derives the kernel's private form of B on every call (for FP8 scales and group sizes
 * other than 32: the exact BF16 expansion, 4 x the bytes of the codes; for asymmetric power-of-two scales of 32-groups:
 * the merged FP6 panel, its block scales and the positions where some row's two scales lie too far apart, about
 * 1.6 bytes per element); for weights that stay, that work can be done once. The product is the same (Sec. 4.3), bit
 * for bit what amxfp4_gemm returns.
 *   amxfp4_weights_prepared_bytes   size of the prepared form of B [N][K]; 0 for the format whose kernel reads B as it
 *                                   is stored (symmetric power-of-two scales of 32-groups), for which the calls below
 *                                   need no buffer and do what amxfp4_gemm does.
 *   amxfp4_prepare_weights          writes it: `prepared` device out, 256-byte aligned, at least that many bytes
 *                                   (AMX_ERR_WORKSPACE otherwise). Depends on fmt, N, K and B only.
 *   amxfp4_gemm_prepared            C = A . B^T with B's prepared form. B_codes / B_scales are still passed: shapes
 *                                   with few rows (M <= 256, see amxfp4_gemm) read B as packed codes and ignore
 *                                   `prepared`. One problem per call (no batch). workspace: at least
 *                                   amxfp4_gemm_prepared_workspace_bytes(), 256-byte aligned (A's expansion only).
 * `prepared` is opaque, valid for this library build, fmt, N and K; the caller owns it and keeps it unchanged while
 * calls that read it are in flight. Other arguments and status codes as amxfp4_gemm.
 */
size_t amxfp4_weights_prepared_bytes(const amx_format_t* fmt, int64_t N, int64_t K);
int amxfp4_prepare_weights(const amx_format_t* fmt, int64_t N, int64_t K, const uint8_t* B_codes,
                           const uint8_t* B_scales, void* prepared, size_t prepared_bytes, void* stream);
size_t amxfp4_gemm_prepared_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K);
int amxfp4_gemm_prepared(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                         const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, const void* prepared,
                         size_t prepared_bytes, float* C, int64_t ldc, void* workspace, size_t workspace_bytes,
                         void* stream);

/*
 * amxfp4_gemm for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation. Same product, same kernels and same results as
 * amxfp4_gemm (bit for bit), but the scratch the kernels need (operand panels, partial tiles) is a static device
 * array inside the library instead of a caller's workspace. The call allocates and frees nothing.
 *   limit      amxfp4_gemm_workspace_bytes(fmt, M, N, K, batch) must not exceed AMXFP4_GEMM_STATIC_BYTES (16 MiB),
 *              else AMX_ERR_WORKSPACE and nothing is launched. That covers the few-rows (decoding) shapes
 *              against any weight matrix, the power-of-two symmetric format up to 5 * 10^8 operand elements (its
 *              scratch is only the re-laid scale bytes, one per 32 elements of either operand), and small
 *              prefill products; large products on the BF16-panel path need amxfp4_gemm.
 *   sharing    every call on a GPU uses that GPU's one array, whose contents are undefined between calls (each call
 *              overwrites what it reads; nothing needs to start at zero). Calls that may execute at the same time on
 *              one GPU (different streams, or replays of two captured graphs) race on it: keep them on one stream.
 *   set-up     the array's device address is looked up on the first call on each GPU (no allocation; each GPU holds
 *              its own copy from the moment the library's code is loaded there until the process ends). Make that
 *              first call outside stream capture.
 * Arguments as amxfp4_gemm, without the workspace.
 */
#define AMXFP4_GEMM_STATIC_BYTES ((size_t)16 << 20)
int amxfp4_gemm_static(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                       const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                       int64_t batch, void* stream);

/*
 * MXFP4 symmetric baseline: the same three calls with `asymmetric` forced to 0 (one scale per group, Sec. 2.1 /
 * Algorithm 1 with the scale format taken from fmt->scale). All other arguments as above.
 */
int mxfp4_quantize(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                   int64_t k_stride, uint8_t* codes, uint8_t* scales, void* stream);
int mxfp4_dequantize(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                     void* out, int32_t out_dtype, void* stream);
int mxfp4_gemm(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
               const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
               int64_t batch, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Double scaling (Sec. 5.3: NVFP4 and its asymmetric variant ANVFP4 combine a tensor-wise FP32 scale with a group-wise
 * FP8-E4M3 scale of 16-element groups; any format of this library can be combined with the tensor-wise scale). The
 * paper names the scheme and gives no arithmetic; this library's definition:
 *   tensor scale   S_t = amax / 2688 in FP32, amax = largest magnitude of the tensor, 2688 = 448 * 6 = the largest
 *                  E4M3 group scale times the largest element, so the group scales use the top of their range;
 *                  never below 2^-96; R_t = 1 / S_t in FP32 (both correctly rounded); an all-zero tensor gives 1, 1.
 *   cast           y = x * R_t in FP32 (one rounding per element), then the group-wise rule at the top of this file
 *                  applied to the y values (real-number quotients y_max / 6 and y / S, sign class = sign bit of x).
 *   value          x_hat = elem * S_group * S_t; the GEMM multiplies the accumulated sum by S_t(A) * S_t(B) in FP32.
 * scale_pair: DEVICE pointer to two floats {S_t, R_t}, 8-byte aligned. amxfp4_tensor_scale writes it (stream-ordered,
 * no host synchronisation; the pair also serves as its scratch), the other calls read it when they execute.
 *
 * amxfp4_tensor_scale: x_bf16 [rows][K] BF16 with rows row_stride apart (K % 8 == 0, row_stride % 8 == 0, 16-byte
 *   aligned base; the maximum does not depend on which axis is later grouped).
 * amxfp4_quantize_scaled / amxfp4_dequantize_scaled (FP32 output only: the product is rounded once) /
 *   amxfp4_gemm_scaled: as the calls without the suffix, plus the scale pair(s). The scaled GEMM always multiplies
 *   exact BF16 operands and needs a workspace of amxfp4_gemm_scaled_workspace_bytes().
 */
int amxfp4_tensor_scale(const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride, float* scale_pair,
                        void* stream);
int amxfp4_quantize_scaled(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                           int64_t k_stride, const float* scale_pair, uint8_t* codes, uint8_t* scales, void* stream);
int amxfp4_dequantize_scaled(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows,
                             int64_t K, const float* scale_pair, float* out, void* stream);
size_t amxfp4_gemm_scaled_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, int64_t batch);
int amxfp4_gemm_scaled(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                       const uint8_t* A_scales, const float* A_scale_pair, const uint8_t* B_codes,
                       const uint8_t* B_scales, const float* B_scale_pair, float* C, int64_t ldc, int64_t batch,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fused quantized attention. The paper quantizes both attention products (Sec. 5.1: Q.K^T and the attention map
 * times V) and defines no fused kernel; this entry point computes them tile by tile without materialising the map.
 * Per query head h (reading key/value head h / (q_heads / kv_heads)) and query i, over key tiles of 32 in ascending
 * order:   s_j = scale * sum_d Q_hat[i, d] K_hat[j, d]   (causal != 0: keys j > i + Sk - Sq are masked; tiles without
 * an unmasked key are skipped);   m' = max(m, max_j s_j);   p_j = exp(s_j - m') (0 when masked);
 * l = l exp(m - m') + sum_j p_j;   p_hat = the 32 values p_j cast as ONE group of `fmt` and dequantized;
 * O = O exp(m - m') + sum_j p_hat_j V_hat[j, :];   finally out[h, i, :] = O / l.   FP32 arithmetic outside the matrix
 * products, whose operands are exact BF16 values. This is not the same number as quantizing the normalised map
 * (amxfp4_gemm on a softmax output): the probabilities are cast relative to the running maximum.
 *   Q_codes/Q_scales   [q_heads][Sq][head_dim] operand cast along head_dim (amxfp4_quantize, k_stride 1).
 *   K_codes/K_scales   [kv_heads][Sk][head_dim] likewise.
 *   V_codes/V_scales   [kv_heads][head_dim][Sk] operand: V^T, cast along the keys (amxfp4_quantize on each head's
 *                      [Sk][head_dim] matrix with row_stride 1, k_stride head_dim).
 *   out                device, [q_heads][Sq][head_dim] floats, 16-byte aligned.
 *   fmt->group_size must be 32 and head_dim 128 or 64 (AMX_ERR_UNSUPPORTED otherwise); Sk % 32 == 0; causal needs
 *   Sk >= Sq.
 *   workspace          at least amxfp4_attention_workspace_bytes() bytes, 256-byte aligned.
 * amxfp4_profile_next_gemm also arms this call (events around the attention kernel proper).
 */
size_t amxfp4_attention_workspace_bytes(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq,
                                        int64_t Sk, int64_t head_dim);
int amxfp4_attention(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                     int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                     const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                     int32_t causal, float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * amxfp4_attention with the output rounded to BF16 (nearest even) and written token-major: out_bf16 [Sq][q_heads *
 * head_dim] BF16 bit patterns, head h in columns h * head_dim .. — the operand of the output projection's cast, bit
 * for bit what amxfp4_merge_heads (amxfp4_layer.h) makes of amxfp4_attention's FP32 result. Everything else as above.
 */
int amxfp4_attention_merged(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                            int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                            const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                            int32_t causal, void* out_bf16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The fused attention for FEW queries against many keys (decoding one or a handful of new tokens against a key / value
 * cache; Sec. 5.1 quantizes both attention products, Sec. 5.2 discusses long context). K and V are read as packed codes
 * and dequantized in registers (no expansion, no panels), the query heads sharing a key / value head are the columns
 * of one wave, and the keys are the parallelism: the Sk / 32 key tiles are cut into key_splits contiguous ranges of
 * ceil((Sk / 32) / key_splits) tiles (the last ones may be shorter or empty); the recurrence of amxfp4_attention runs
 * over each range on its own, from m = -inf, l = 0, O = 0, giving (m_c, l_c, O_c), and
 *     m* = max_c m_c;   out[i, :] = sum_c O_c exp(m_c - m*) / sum_c l_c exp(m_c - m*)
 * (ranges in which the query sees no key left out). The probabilities of a range are cast against that range's own
 * running maximum, so the result depends on key_splits; key_splits = 1 is amxfp4_attention's definition.
 *   limits     (q_heads / kv_heads) * Sq <= 32 (AMX_ERR_UNSUPPORTED beyond: use amxfp4_attention); group_size 32;
 *              head_dim 128 or 64; 1 <= key_splits <= min(1024, Sk / 32); kv_heads <= 65535. A batch of sequences of
 *              equal length is a larger number of heads.
 *   speed      with Sk % 256 == 0 a wave fetches V in chunks of 8 key tiles; ranges of whole chunks (key_splits
 *              dividing Sk / 256) read every byte of V once.
 *   workspace  at least amxfp4_attention_decode_workspace_bytes() bytes, 256-byte aligned (the ranges' partial results:
 *              kv_heads * key_splits * 32 * (head_dim + 2) floats).
 * Other arguments, layouts and status codes as amxfp4_attention; out is FP32 [q_heads][Sq][head_dim].
 */
size_t amxfp4_attention_decode_workspace_bytes(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq,
                                               int64_t Sk, int64_t head_dim, int64_t key_splits);
int amxfp4_attention_decode(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                            int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                            const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                            int32_t causal, int64_t key_splits, float* out, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * Measurement aid (not part of the method): arms a pair of caller-owned hipEvent_t (passed as void*) for the NEXT
 * amxfp4_gemm / mxfp4_gemm call made on this host thread. That call records `start` on its stream immediately before
 * and `stop` immediately after the launch of its matrix-multiply kernel (the MFMA main loop, excluding the operand
 * re-layout kernels that precede it), then disarms itself. Pass NULL, NULL to disarm. Returns AMX_OK.
 */
int amxfp4_profile_next_gemm(void* start_event, void* stop_event);

/*
 * Per-call kernel choice for amxfp4_gemm_ex (tuning and test aid, not part of the method). Several kernels compute the
 * same product (Sec. 4.3) for some formats; they differ in where the operands are dequantized and hence in speed and
 * workspace, not in the result beyond the FP32 summation order. All fields 0 = what amxfp4_gemm does. The library
 * keeps no process-wide choice and reads no environment variable: the options of a call are the whole story, and
 * amxfp4_gemm_workspace_bytes_ex is a pure function of its arguments.
 *   e5m2_kernel   FP8-E5M2 scales, groups of 32 (Sec. 4.2 "FP8"):
 *                   AMX_E5M2_PANEL   both operands expanded to BF16 panels in the workspace, BF16 MFMA (any K);
 *                   AMX_E5M2_HYBRID  A expanded to an FP16 panel, B dequantized inside the FP16 MFMA kernel (K % 128 == 0);
 *                   AMX_E5M2_FUSED   both operands dequantized inside the kernel, no workspace (K % 128 == 0).
 *   pot_kernel    asymmetric power-of-two scales, groups of 32 (Sec. 4.2 "PoT"):
 *                   AMX_POT_MERGED_FP6  each group merged into ONE FP6 (E3M2) operand block, elem * 2^(s_class - anchor),
 *                                    which is exact while the two scale exponents of the group differ by at most 5;
 *                                    a group position where some row's scales lie further apart is written twice
 *                                    along K, once per sign class, so nothing is ever rounded or dropped except a
 *                                    class whose scale byte is 0 (2^-127: what the cast writes for a class without
 *                                    elements). Block-scaled MFMA at the FP4 rate (default; any K; workspace sized for
 *                                    the worst case, every position split in both operands: about 3 bytes per element);
 *                   AMX_POT_SPLIT_FP4   each operand split by sign into two MXFP4 operands, four block-scaled FP4 MFMAs
 *                                    per block (exact; K % 128 == 0; workspace: the re-laid scale bytes only);
 *                   AMX_POT_MERGED_FP8  each group merged into E5M2 elements with one anchor scale max(s_p, s_n): one
 *                                    block-scaled FP8 MFMA per block (any K; 1 byte per element of workspace). An
 *                                    element whose class scale lies more than 2^13 below the anchor is flushed to zero
 *                                    (less than 1e-4 of its group's largest magnitude), and the instruction adds the
 *                                    products of a block in a fixed-point window below the largest product, so a sum
 *                                    whose classes cancel can carry an absolute error of about 2^-22 of that largest
 *                                    product: far inside the 1e-3 tolerance in norm, not bit-exact.
 *   tile          workgroup tile of the BF16-panel kernel: AMX_TILE_AUTO (a cost model over the shape), or
 *                 AMX_TILE_256x256 / AMX_TILE_256x128 / AMX_TILE_64x256 on any shape.
 *   few_rows      the kernel that reads B as packed codes (M <= 256, or <= 768 against a large B; K % 256 == 0):
 *                 0 = use it where it applies, -1 = never, n > 0 = use it where it applies with n outer K slices
 *                 (at most 16 and at most K / 256).
 * A kernel that does not take the shape or format falls back to the default one. Unknown values: AMX_ERR_INVALID_ARG.
 */
enum { AMX_E5M2_PANEL = 0, AMX_E5M2_HYBRID = 1, AMX_E5M2_FUSED = 2 };
enum { AMX_POT_MERGED_FP6 = 0, AMX_POT_SPLIT_FP4 = 1, AMX_POT_MERGED_FP8 = 2 };
enum { AMX_TILE_AUTO = 0, AMX_TILE_256x256 = 1, AMX_TILE_256x128 = 2, AMX_TILE_64x256 = 3 };
typedef struct {
  int32_t e5m2_kernel;
  int32_t pot_kernel;
  int32_t tile;
  int32_t few_rows;
} amx_gemm_options_t;

/* amxfp4_gemm_workspace_bytes / amxfp4_gemm with the kernel chosen by `opts` (HOST pointer; NULL = all defaults). */
size_t amxfp4_gemm_workspace_bytes_ex(const amx_format_t* fmt, const amx_gemm_options_t* opts, int64_t M, int64_t N,
                                      int64_t K, int64_t batch);
int amxfp4_gemm_ex(const amx_format_t* fmt, const amx_gemm_options_t* opts, int64_t M, int64_t N, int64_t K,
                   const uint8_t* A_codes, const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales,
                   float* C, int64_t ldc, int64_t batch, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aids (not part of the method): what this machine sustains on the resources that bound the path.
 *
 * amxfp4_peak_mfma runs a register-resident loop of matrix instructions (512 workgroups of 4 waves, 16 independent
 * 32x32 accumulator tiles per wave, `iterations` rounds, no memory traffic inside the loop) and writes the number of
 * floating-point operations it performs to the HOST double *flops; the caller times the call on `stream`.
 *   mfma       0 = BF16 32x32x16, 1 = block-scaled FP8 (E5M2) 32x32x64, 2 = block-scaled FP4 32x32x64 (unit scales),
 *              3 = FP16 32x32x16, 4 = block-scaled FP6 (E3M2) 32x32x64.
 *   operand    device, 16384 bytes, 16-byte aligned: lane t of a workgroup takes bytes 64t .. 64t+31 as its A and
 *              64t+32 .. 64t+63 as its B operand registers (BF16, FP16 and FP4 use the first 16 of each, FP6 the
 *              first 24). The sustained
 *              rate depends on these bits (clock management), so pass zeros for the best case and a slice of a real
 *              operand for the realistic one.
 *   sink       device out, 512 * 256 floats (contents meaningless).
 * amxfp4_peak_copy copies `bytes` (a multiple of 16; both buffers device, 16-byte aligned, not overlapping) with
 * plain 128-bit loads and stores: a streaming-bandwidth reference that moves 2 * bytes.
 */
int amxfp4_peak_mfma(int32_t mfma, const void* operand, int32_t iterations, float* sink, double* flops,
                     void* stream);
int amxfp4_peak_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AMXFP4_H */
