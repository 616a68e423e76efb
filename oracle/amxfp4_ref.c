/*
 * amxfp4_ref.c — the CPU ORACLE for AMXFP4 / MXFP4 quantization, dequantization and the quantized GEMM.
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, scalar implementation that follows the paper's steps in the
 * paper's order; only tests, the smoke check and the benchmark's cpu_baseline leg may call it. It shares no code,
 * header, table or helper with the GPU library, and the GPU library never calls it.
 *
 * What it follows:
 *   - grouping along the last (contraction) axis, group size 32 by default, -1 = the whole row (Sec. 2.1;
 *     Appendix B code example, which uses one group per row);
 *   - MX quantization (Appendix B, Algorithm 1): shared scale from the group's largest magnitude, then each element
 *     divided by the scale, rounded onto the element grid and clamped to the largest normal;
 *   - asymmetric FP (Sec. 4.1 "AsymFP", Sec. 4.2 Eq. 1): positive and negative elements each get their own shared
 *     scale, derived from the largest positive value and the largest |negative value| of the group;
 *   - FP8 E5M2 shared scale (Sec. 4.2 "FP8"): the scale is amax / 6 (6 = largest E2M1 magnitude) rounded to the
 *     nearest E5M2 value; power-of-two scales: 2^(floor(log2 amax) - 2) (Algorithm 1, emax_elem = 2), or with the
 *     exponent rounded (Appendix B "Floor vs. Round");
 *   - the product of two AMXFP4 numbers uses the scales selected by their two signs (Sec. 4.3); the GEMM is the
 *     plain sum over k of those products, accumulated in double, rounded once to float;
 *   - double scaling (Sec. 5.3: NVFP4 and its asymmetric variant ANVFP4 put a tensor-wise FP32 scale under a
 *     group-wise FP8 E4M3 scale of 16-element groups): the *_scaled functions below. The paper names the scheme and
 *     gives no arithmetic for it; the reading taken here is written at those functions       — parity unpinned
 *
 * Readings of points the paper leaves open (each is repeated in the repository's design notes):
 *   - ties in both roundings go to the even code / even mantissa (OCP MX default)               — parity unpinned
 *   - an empty sign class, or a scale that rounds to zero, stores scale byte 0 and magnitude 0   — parity unpinned
 *   - E5M2 scale saturates at 57344; E8M0 byte is clamped to [0, 254]                            — parity unpinned
 *   - the sign bit of a code is the IEEE sign bit of the input, also for magnitude 0             — parity unpinned
 *   - exponent rounding for the power-of-two scale: exponent + 1 when the significand of amax exceeds sqrt(2)
 *     (round(log2 amax)); the paper does not state the rule                                      — parity unpinned
 *   - byte/nibble layout of codes and scales (the paper's figure is not reproduced in its text)  — parity unpinned
 * Everything else is pinned by tests that do not use this file's formulas (printed example of Appendix B,
 * brute-force nearest-value searches in exact rational arithmetic, algebraic invariants).
 *
 * All arithmetic is on doubles holding exact values: BF16 inputs, scales and thresholds are dyadic rationals with a
 * handful of significant bits, so every comparison below is exact.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t group_size; /* -1 = whole row */
  int32_t elem;       /* 0 = FP4 E2M1 */
  int32_t scale;      /* 0 = E8M0 floor, 1 = E8M0 round, 2 = FP8 E5M2, 3 = FP8 E4M3 */
  int32_t asymmetric; /* 1 = two scales per group (positive, negative), 0 = one */
} ref_format_t;

enum { SC_E8M0_FLOOR = 0, SC_E8M0_ROUND = 1, SC_E5M2 = 2, SC_E4M3 = 3 };

/* E2M1 magnitudes by 3-bit code e1 e0 m: exponent bias 1, code 1 is the subnormal 0.5 (Sec. 2.1). */
static const double kE2M1[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

static float bf16_to_float(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* ---------------------------------------------------------------- scales ---------------------------------- */

/* Value of a scale byte. */
double amxfp4_scale_decode_ref(int32_t kind, uint8_t byte) {
  if (kind == SC_E8M0_FLOOR || kind == SC_E8M0_ROUND) return ldexp(1.0, (int)byte - 127);
  if (kind == SC_E5M2) {
    int e = (byte >> 2) & 31, m = byte & 3;
    return e == 0 ? ldexp((double)m, -16) : ldexp(1.0 + m / 4.0, e - 15);
  }
  /* E4M3: bias 7, subnormals m * 2^-9 */
  int e = (byte >> 3) & 15, m = byte & 7;
  return e == 0 ? ldexp((double)m, -9) : ldexp(1.0 + m / 8.0, e - 7);
}

/* Round q >= 0 to the nearest value of a small float format with `mbits` mantissa bits, minimum normal exponent
 * `emin`, ties to even, saturating at `vmax`. Returns the rounded value. */
static double round_to_minifloat(double q, int mbits, int emin, double vmax) {
  if (q <= 0.0) return 0.0;
  int ex;
  (void)frexp(q, &ex); /* q = f * 2^ex, f in [0.5, 1)  =>  floor(log2 q) = ex - 1 */
  int e = ex - 1;
  if (e < emin) e = emin;                 /* subnormal range shares the spacing of the lowest binade */
  double quantum = ldexp(1.0, e - mbits); /* spacing of representable values around q */
  double n = nearbyint(q / quantum);      /* default rounding mode: nearest, ties to even */
  double v = n * quantum;
  return v > vmax ? vmax : v;
}

/* Encode a non-negative representable value of the given FP8 scale format into its byte. */
static uint8_t minifloat_byte(double v, int mbits, int bias, int emin) {
  if (v == 0.0) return 0;
  int ex;
  double f = frexp(v, &ex);
  int e = ex - 1;
  if (e < emin) { /* subnormal: v = m * 2^(emin - mbits) */
    return (uint8_t)lrint(ldexp(v, mbits - emin));
  }
  int m = (int)lrint((f * 2.0 - 1.0) * (double)(1 << mbits));
  return (uint8_t)(((e + bias) << mbits) | m);
}

/* Shared scale byte for a sign class whose largest magnitude is amax (>= 0). */
uint8_t amxfp4_scale_encode_ref(int32_t kind, double amax) {
  if (!(amax > 0.0)) return 0;
  if (kind == SC_E8M0_FLOOR || kind == SC_E8M0_ROUND) {
    int ex;
    double f = frexp(amax, &ex); /* amax = f * 2^ex, f in [0.5,1): significand 2f in [1,2), exponent ex-1 */
    int e = ex - 1;
    if (kind == SC_E8M0_ROUND && (2.0 * f) * (2.0 * f) > 2.0) e += 1; /* round(log2 amax) */
    int byte = e - 2 + 127;                                          /* emax_elem = 2 (Algorithm 1) */
    if (byte < 0) byte = 0;
    if (byte > 254) byte = 254;
    return (uint8_t)byte;
  }
  double q = amax / 6.0; /* 6 = largest E2M1 magnitude */
  if (kind == SC_E5M2) return minifloat_byte(round_to_minifloat(q, 2, -14, 57344.0), 2, 15, -14);
  return minifloat_byte(round_to_minifloat(q, 3, -6, 448.0), 3, 7, -6);
}

/* ---------------------------------------------------------------- elements -------------------------------- */

/* 3-bit magnitude code of |x| under scale S: nearest E2M1 value to min(|x|/S, 6), ties to the even code.
 * The comparison |x|/S vs t is done as |x| vs t*S, exact in double. */
uint8_t amxfp4_elem_encode_ref(double absx, double S) {
  if (!(S > 0.0)) return 0;
  uint8_t c = 0;
  if (absx > 0.25 * S) c = 1;  /* tie 0.25 -> 0   (code 0, even) */
  if (absx >= 0.75 * S) c = 2; /* tie 0.75 -> 1.0 (code 2, even) */
  if (absx > 1.25 * S) c = 3;  /* tie 1.25 -> 1.0 (code 2) */
  if (absx >= 1.75 * S) c = 4; /* tie 1.75 -> 2.0 (code 4) */
  if (absx > 2.5 * S) c = 5;   /* tie 2.5  -> 2.0 (code 4) */
  if (absx >= 3.5 * S) c = 6;  /* tie 3.5  -> 4.0 (code 6) */
  if (absx > 5.0 * S) c = 7;   /* tie 5    -> 4.0 (code 6); everything above saturates at 6 */
  return c;
}

/* ---------------------------------------------------------------- quantize -------------------------------- */

static int check_format(const ref_format_t* f, int64_t K, int64_t* gs_out) {
  if (!f || f->elem != 0 || f->scale < 0 || f->scale > 3) return -1;
  int64_t gs = f->group_size == -1 ? K : f->group_size;
  if (gs <= 0 || K <= 0 || K % gs != 0 || K % 2 != 0) return -1;
  *gs_out = gs;
  return 0;
}

/*
 * Tensor-wise scale of the double-scaling scheme (Sec. 5.3). Reading: the tensor scale maps the tensor's largest
 * magnitude onto the largest value a group scale times an element can express, 448 * 6 = 2688 (448 = largest E4M3
 * value, 6 = largest E2M1 value), so that the group scales use the top of the E4M3 range:
 *   out[0] = S_t = float(amax_tensor) / 2688 in single precision, not below 2^-96 (so that 1 / S_t is finite);
 *   out[1] = R_t = 1 / S_t in single precision, the factor the cast multiplies by.
 * An all-zero tensor gives S_t = R_t = 1. x_hat = elem * S_group * S_t.
 */
int amxfp4_tensor_scale_ref(const uint16_t* x_bf16, int64_t rows, int64_t K, int64_t row_stride, int64_t k_stride,
                            float* out) {
  if (!x_bf16 || !out || rows <= 0 || K <= 0) return -1;
  float amax = 0.0f;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t k = 0; k < K; ++k) {
      float v = fabsf(bf16_to_float(x_bf16[r * row_stride + k * k_stride]));
      if (v > amax) amax = v;
    }
  if (amax == 0.0f) {
    out[0] = out[1] = 1.0f;
    return 0;
  }
  volatile float st = amax / 2688.0f; /* volatile: one rounding to single precision, no wider intermediate */
  if (st < 0x1p-96f) st = 0x1p-96f;
  volatile float rt = 1.0f / st;
  out[0] = st;
  out[1] = rt;
  return 0;
}

/*
 * One group: y[0..gs) are the values to quantize (single-precision numbers, of which BF16 inputs are a subset); the
 * sign class of an element is its IEEE sign bit. Writes the group's scale byte(s) to sc and ORs the element codes
 * into the (pre-zeroed) code row at element positions k0, k0 + 1, ...
 */
static void quantize_group(const ref_format_t* fmt, const float* y, int64_t gs, uint8_t* code_row, int64_t k0,
                           uint8_t* sc) {
  /* step 1-2: largest positive value and largest |negative value| of the group */
  double amax_p = 0.0, amax_n = 0.0;
  for (int64_t i = 0; i < gs; ++i) {
    double v = (double)y[i];
    if (signbit(y[i])) {
      if (-v > amax_n) amax_n = -v;
    } else {
      if (v > amax_p) amax_p = v;
    }
  }
  if (!fmt->asymmetric) amax_p = amax_n = (amax_p > amax_n ? amax_p : amax_n);
  /* step 3: shared scale(s) */
  uint8_t sb_p = amxfp4_scale_encode_ref(fmt->scale, amax_p);
  uint8_t sb_n = amxfp4_scale_encode_ref(fmt->scale, amax_n);
  sc[0] = sb_p;
  if (fmt->asymmetric) sc[1] = sb_n;
  /* a class with no magnitude stores byte 0 and quantizes to magnitude 0; an FP8 scale that rounded to zero
   * decodes to 0 and does the same */
  double S_p = amax_p > 0.0 ? amxfp4_scale_decode_ref(fmt->scale, sb_p) : 0.0;
  double S_n = amax_n > 0.0 ? amxfp4_scale_decode_ref(fmt->scale, sb_n) : 0.0;
  /* step 4-5: element codes, two per byte, low nibble first */
  for (int64_t i = 0; i < gs; ++i) {
    int neg = signbit(y[i]) != 0;
    double a = fabs((double)y[i]);
    uint8_t code = (uint8_t)((neg << 3) | amxfp4_elem_encode_ref(a, neg ? S_n : S_p));
    int64_t k = k0 + i;
    code_row[k / 2] |= (uint8_t)(code << (4 * (k & 1)));
  }
}

/*
 * Direct cast with a tensor-wise scale (Sec. 5.3 double scaling; tensor_rcp = 1 is the plain cast of Algorithm 1 /
 * Eq. 1, for which the multiplication below is exact). Reading: every element is first multiplied by R_t in single
 * precision, y = float(x * R_t) (one rounding), and the group-wise algorithm then runs on the y values exactly as
 * it runs on BF16 values (the multiplication by R_t > 0 keeps the sign bit, also of zeros).
 */
int amxfp4_quantize_scaled_ref(const ref_format_t* fmt, const uint16_t* x_bf16, int64_t rows, int64_t K,
                               int64_t row_stride, int64_t k_stride, float tensor_rcp, uint8_t* codes,
                               uint8_t* scales) {
  int64_t gs;
  if (check_format(fmt, K, &gs) || !x_bf16 || !codes || !scales || rows <= 0 || !(tensor_rcp > 0.0f)) return -1;
  const int64_t G = K / gs;
  const int ns = fmt->asymmetric ? 2 : 1;
  memset(codes, 0, (size_t)(rows * K / 2));
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    float* y = (float*)malloc(sizeof(float) * (size_t)gs);
    for (int64_t g = 0; g < G; ++g) {
      const uint16_t* xg = x_bf16 + r * row_stride + g * gs * k_stride;
      for (int64_t i = 0; i < gs; ++i) {
        volatile float yi = bf16_to_float(xg[i * k_stride]) * tensor_rcp; /* one rounding to single precision */
        y[i] = yi;
      }
      quantize_group(fmt, y, gs, codes + r * (K / 2), g * gs, scales + (r * G + g) * ns);
    }
    free(y);
  }
  return 0;
}

/* The same group-wise cast of single-precision values y [rows][K] (contiguous). Used where the values to quantize
 * are produced in single precision rather than read as BF16 (the attention probabilities of a fused softmax). */
int amxfp4_quantize_f32_ref(const ref_format_t* fmt, const float* y, int64_t rows, int64_t K, uint8_t* codes,
                            uint8_t* scales) {
  int64_t gs;
  if (check_format(fmt, K, &gs) || !y || !codes || !scales || rows <= 0) return -1;
  const int64_t G = K / gs;
  const int ns = fmt->asymmetric ? 2 : 1;
  memset(codes, 0, (size_t)(rows * K / 2));
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t g = 0; g < G; ++g)
      quantize_group(fmt, y + r * K + g * gs, gs, codes + r * (K / 2), g * gs, scales + (r * G + g) * ns);
  return 0;
}

int amxfp4_quantize_ref(const ref_format_t* fmt, const uint16_t* x_bf16, int64_t rows, int64_t K,
                        int64_t row_stride, int64_t k_stride, uint8_t* codes, uint8_t* scales) {
  return amxfp4_quantize_scaled_ref(fmt, x_bf16, rows, K, row_stride, k_stride, 1.0f, codes, scales);
}

/* ---------------------------------------------------------------- dequantize ------------------------------ */

/* x_hat = (-1)^s * elem * S_class (Eq. 1). out is row-major [rows][K] doubles. */
int amxfp4_dequantize_ref(const ref_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows,
                          int64_t K, double* out) {
  int64_t gs;
  if (check_format(fmt, K, &gs) || !codes || !scales || !out || rows <= 0) return -1;
  const int64_t G = K / gs;
  const int ns = fmt->asymmetric ? 2 : 1;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    for (int64_t k = 0; k < K; ++k) {
      uint8_t byte = codes[r * (K / 2) + k / 2];
      uint8_t code = (byte >> (4 * (k & 1))) & 15;
      int neg = code >> 3;
      const uint8_t* sc = scales + (r * G + k / gs) * ns;
      uint8_t sb = fmt->asymmetric ? sc[neg] : sc[0];
      double S = amxfp4_scale_decode_ref(fmt->scale, sb);
      double v = kE2M1[code & 7] * S;
      out[r * K + k] = neg ? -v : v;
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- GEMM ------------------------------------ */

/* C[b][i][j] = float( sum_k A_hat[b][i][k] * B_hat[b][j][k] ), sum in double in index order (Sec. 4.3). */
/* With tensor-wise scales (Sec. 5.3): x_hat = elem * S_group * S_t, so the sum is multiplied by the two tensor
 * scales (in double) before the single rounding to float. */
int amxfp4_gemm_scaled_ref(const ref_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                           const uint8_t* A_scales, float A_tensor_scale, const uint8_t* B_codes,
                           const uint8_t* B_scales, float B_tensor_scale, float* C, int64_t ldc, int64_t batch) {
  int64_t gs;
  if (check_format(fmt, K, &gs) || !A_codes || !A_scales || !B_codes || !B_scales || !C || M <= 0 || N <= 0 ||
      ldc < N || batch <= 0)
    return -1;
  const int64_t G = K / gs;
  const int ns = fmt->asymmetric ? 2 : 1;
  double* Ah = (double*)malloc(sizeof(double) * (size_t)(M * K));
  double* Bh = (double*)malloc(sizeof(double) * (size_t)(N * K));
  if (!Ah || !Bh) {
    free(Ah);
    free(Bh);
    return -2;
  }
  for (int64_t b = 0; b < batch; ++b) {
    amxfp4_dequantize_ref(fmt, A_codes + b * M * (K / 2), A_scales + b * M * G * ns, M, K, Ah);
    amxfp4_dequantize_ref(fmt, B_codes + b * N * (K / 2), B_scales + b * N * G * ns, N, K, Bh);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
      for (int64_t j = 0; j < N; ++j) {
        double acc = 0.0;
        const double* a = Ah + i * K;
        const double* bb = Bh + j * K;
        for (int64_t k = 0; k < K; ++k) acc += a[k] * bb[k];
        C[(b * M + i) * ldc + j] = (float)(acc * (double)A_tensor_scale * (double)B_tensor_scale);
      }
    }
  }
  free(Ah);
  free(Bh);
  return 0;
}

int amxfp4_gemm_ref(const ref_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                    const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                    int64_t batch) {
  return amxfp4_gemm_scaled_ref(fmt, M, N, K, A_codes, A_scales, 1.0f, B_codes, B_scales, 1.0f, C, ldc, batch);
}

/* Number of threads the loops above use. */
int amxfp4_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
