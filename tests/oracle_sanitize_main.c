/* Driver for the sanitizer run of the oracle (tests/test_oracle_sanitizers.py compiles this file together with
 * oracle/amxfp4_ref.c under AddressSanitizer and UndefinedBehaviorSanitizer and runs it): every entry point on
 * exact-size heap buffers, all scale formats, both symmetries, group sizes 16 / 32 / 64 / whole row, strided input,
 * ragged shapes, a batch, zero and extreme inputs. Any read or write past a buffer, and any undefined operation, aborts
 * the program; it prints "ok" and returns 0 otherwise. Results are checked elsewhere. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t group_size, elem, scale, asymmetric;
} ref_format_t;

int amxfp4_tensor_scale_ref(const uint16_t* x_bf16, int64_t rows, int64_t K, int64_t row_stride, int64_t k_stride,
                            float* pair);
int amxfp4_quantize_scaled_ref(const ref_format_t* fmt, const uint16_t* x_bf16, int64_t rows, int64_t K,
                               int64_t row_stride, int64_t k_stride, float tensor_rcp, uint8_t* codes, uint8_t* scales);
int amxfp4_quantize_f32_ref(const ref_format_t* fmt, const float* y, int64_t rows, int64_t K, uint8_t* codes,
                            uint8_t* scales);
int amxfp4_quantize_ref(const ref_format_t* fmt, const uint16_t* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                        int64_t k_stride, uint8_t* codes, uint8_t* scales);
int amxfp4_dequantize_ref(const ref_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                          double* out);
int amxfp4_gemm_scaled_ref(const ref_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                           const uint8_t* A_scales, float A_tensor, const uint8_t* B_codes, const uint8_t* B_scales,
                           float B_tensor, float* C, int64_t ldc, int64_t batch);
int amxfp4_gemm_ref(const ref_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                    const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                    int64_t batch);

static uint32_t state = 12345u;
static uint32_t next_u32(void) {
  state = state * 1664525u + 1013904223u;
  return state;
}
/* BF16 bit patterns: finite values over the whole exponent range, zeros, both signs */
static uint16_t random_bf16(int kind) {
  uint32_t r = next_u32() >> 8;
  uint16_t sign = (uint16_t)((r & 1u) << 15), mant = (uint16_t)((r >> 1) & 0x7Fu);
  if (kind == 0) return sign;                                                    /* zeros */
  if (kind == 1) return (uint16_t)(sign | ((100u + (r >> 8) % 56u) << 7) | mant); /* moderate */
  return (uint16_t)(sign | (((r >> 8) % 255u) << 7) | mant);                      /* any finite, subnormals included */
}

static void fail(const char* what) {
  fprintf(stderr, "oracle call failed: %s\n", what);
  exit(1);
}

static void run(int64_t M, int64_t N, int64_t K, int32_t gs, int32_t scale, int32_t asym, int kind, int64_t batch) {
  const ref_format_t fmt = {gs, 0, scale, asym};
  const int64_t g = gs > 0 ? gs : K, G = K / g, ns = asym ? 2 : 1;
  uint16_t* a = malloc((size_t)(batch * M * K) * 2);
  uint16_t* b = malloc((size_t)(batch * N * K) * 2);
  for (int64_t i = 0; i < batch * M * K; ++i) a[i] = random_bf16(kind);
  for (int64_t i = 0; i < batch * N * K; ++i) b[i] = random_bf16(kind == 2 ? 1 : kind);
  uint8_t* ac = malloc((size_t)(batch * M * K / 2));
  uint8_t* as = malloc((size_t)(batch * M * G * ns));
  uint8_t* bc = malloc((size_t)(batch * N * K / 2));
  uint8_t* bs = malloc((size_t)(batch * N * G * ns));
  if (amxfp4_quantize_ref(&fmt, a, batch * M, K, K, 1, ac, as)) fail("quantize A");
  if (amxfp4_quantize_ref(&fmt, b, batch * N, K, K, 1, bc, bs)) fail("quantize B");
  double* d = malloc((size_t)(batch * M * K) * 8);
  if (amxfp4_dequantize_ref(&fmt, ac, as, batch * M, K, d)) fail("dequantize");
  const int64_t ldc = N + 3;
  float* c = malloc((size_t)(batch * M * ldc) * 4);
  if (amxfp4_gemm_ref(&fmt, M, N, K, ac, as, bc, bs, c, ldc, batch)) fail("gemm");
  /* tensor-wise scale on top (Sec. 5.3), and the single-precision cast */
  float pair[2];
  if (amxfp4_tensor_scale_ref(a, batch * M, K, K, 1, pair)) fail("tensor_scale");
  if (amxfp4_quantize_scaled_ref(&fmt, a, batch * M, K, K, 1, pair[1], ac, as)) fail("quantize_scaled");
  if (amxfp4_gemm_scaled_ref(&fmt, M, N, K, ac, as, pair[0], bc, bs, 1.0f, c, ldc, batch)) fail("gemm_scaled");
  float* y = malloc((size_t)(M * K) * 4);
  for (int64_t i = 0; i < M * K; ++i) y[i] = (float)(next_u32() >> 8) / 16777216.0f;
  if (amxfp4_quantize_f32_ref(&fmt, y, M, K, ac, as)) fail("quantize_f32");
  /* groups down the columns of a [K][M] matrix: row_stride 1, k_stride M (the V operand of the attention) */
  if (batch == 1 && amxfp4_quantize_ref(&fmt, a, M, K, 1, M, ac, as)) fail("quantize strided");
  free(a), free(b), free(ac), free(as), free(bc), free(bs), free(d), free(c), free(y);
}

int main(void) {
  const int32_t scales[4] = {0, 1, 2, 3};
  for (int s = 0; s < 4; ++s)
    for (int32_t asym = 0; asym < 2; ++asym)
      for (int kind = 0; kind < 3; ++kind) {
        run(5, 7, 64, 32, scales[s], asym, kind, 1);
        run(3, 2, 96, 16, scales[s], asym, kind, 2);
        run(2, 9, 128, 64, scales[s], asym, kind, 1);
        run(4, 3, 40, -1, scales[s], asym, kind, 1);
        run(1, 1, 32, 32, scales[s], asym, kind, 3);
      }
  puts("ok");
  return 0;
}
