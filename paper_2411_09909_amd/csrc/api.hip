// C ABI of libamxfp4 (declared in include/amxfp4.h): host-side validation and dispatch. No arithmetic of the
// method happens here; every step runs in the kernels of cast.hip / gemm_*.hip.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/amxfp4.h"
#include "../../include/amxfp4_layer.h"
#include "kernels.h"

// Scratch of amxfp4_gemm_static, the entry point for callers that cannot allocate: device memory that exists from
// the moment the code object is loaded on a GPU until the process ends, one copy per GPU. Host code never uses this
// name as an address (it is a host-side stand-in): static_scratch() below asks the runtime for the device address.
constexpr size_t kStaticScratchBytes = AMXFP4_GEMM_STATIC_BYTES;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[256] = "no error";
thread_local amx::KernelTimer g_timer;  // armed by amxfp4_profile_next_gemm, consumed by the next GEMM call

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// Size limits (stated in include/amxfp4.h): K of any operand, rows of a cast, rows of a GEMM operand, batch entries.
constexpr int64_t kMaxK = int64_t(1) << 20;
constexpr int64_t kMaxCastRows = (int64_t(1) << 31) - 1;
constexpr int64_t kMaxStridedRows = 65535 * 256;
constexpr int64_t kMaxGemmRows = (int64_t(1) << 21) - 256;
constexpr int64_t kMaxBatch = 65535;
constexpr int64_t kMaxLdc = int64_t(1) << 22;  // the kernels address a wave's window of C with 32-bit byte offsets

// Validates a format for the GPU library. Returns AMX_OK or a negative status (message set). whole_row_ok: the caller
// implements one group per row (group_size -1): the contiguous cast, the dequantization and the GEMM entry points.
int check_format(const amx_format_t* f, bool whole_row_ok = false) {
  if (!f) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (f->elem != AMX_ELEM_FP4_E2M1) return fail(AMX_ERR_INVALID_ARG, "unknown element format %d", f->elem);
  if (f->scale < AMX_SCALE_E8M0_FLOOR || f->scale > AMX_SCALE_FP8_E4M3)
    return fail(AMX_ERR_INVALID_ARG, "unknown scale format %d", f->scale);
  if (f->asymmetric != 0 && f->asymmetric != 1) return fail(AMX_ERR_INVALID_ARG, "asymmetric must be 0 or 1");
  if (f->group_size == 0 || f->group_size < -1) return fail(AMX_ERR_INVALID_ARG, "bad group_size %d", f->group_size);
  if (f->group_size == -1) {
    if (!whole_row_ok)
      return fail(AMX_ERR_UNSUPPORTED, "whole-row groups (group_size -1) are implemented by the contiguous cast, the "
                                       "dequantization and the GEMM entry points only");
    return AMX_OK;
  }
  if (f->group_size != 16 && f->group_size != 32 && f->group_size != 64 && f->group_size != 128)
    return fail(AMX_ERR_UNSUPPORTED, "the GPU library implements group sizes 16, 32, 64, 128 and -1 (got %d)",
                f->group_size);
  return AMX_OK;
}

int check_shape(const amx_format_t& f, int64_t rows, int64_t K) {
  if (rows <= 0 || K <= 0) return fail(AMX_ERR_INVALID_ARG, "rows and K must be positive (got %lld, %lld)",
                                       (long long)rows, (long long)K);
  if (!amx::group_divides(K, f.group_size) || K % 32 != 0)
    return fail(AMX_ERR_INVALID_ARG, "K = %lld is not a multiple of the group size %d and of 32", (long long)K,
                f.group_size);
  // launch grids and 32-bit offsets inside the kernels are laid out for these bounds
  if (K > kMaxK) return fail(AMX_ERR_INVALID_ARG, "K = %lld exceeds the supported maximum %lld", (long long)K, (long long)kMaxK);
  if (rows > kMaxCastRows)
    return fail(AMX_ERR_INVALID_ARG, "rows = %lld exceeds the supported maximum %lld", (long long)rows, (long long)kMaxCastRows);
  return AMX_OK;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int hip_fail(hipError_t e, const char* what) {
  return fail(AMX_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Device address of `scratch` on the current GPU, looked up once per device (every GPU holds its own copy of the
// array at its own address) and kept: a cache of addresses that never change, not a setting.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(AMX_ERR_UNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AMX_OK;
}

}  // namespace

namespace amx {
// the same thread-local status message for the entry points defined in other files
int report_error(int code, const char* msg) { return fail(code, "%s", msg); }
int report_hip_error(hipError_t e, const char* what) { return hip_fail(e, what); }
}  // namespace amx

namespace {

int quantize_impl(amx_format_t f, const void* x, int64_t batch, int64_t batch_stride, int64_t rows, int64_t K,
                  int64_t row_stride, int64_t k_stride, const float* tensor_pair, uint8_t* codes, uint8_t* scales,
                  void* stream) {
  if (int rc = check_format(&f, k_stride == 1)) return rc;
  if (int rc = check_shape(f, rows, K)) return rc;
  if (batch < 1 || batch > kMaxBatch)
    return fail(AMX_ERR_INVALID_ARG, "batch = %lld outside 1 .. %lld", (long long)batch, (long long)kMaxBatch);
  if (batch > 1 && batch_stride < 0) return fail(AMX_ERR_INVALID_ARG, "negative batch_stride");
  if (!x || !codes || !scales) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(codes, 16) || !aligned(scales, 4)) return fail(AMX_ERR_INVALID_ARG, "codes need 16-byte, scales 4-byte alignment");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const uint16_t* xb = reinterpret_cast<const uint16_t*>(x);
  if (k_stride == 1) {
    if (row_stride < K || row_stride % 8 != 0 || !aligned(x, 16) || (batch > 1 && batch_stride % 8 != 0))
      return fail(AMX_ERR_INVALID_ARG, "contiguous cast needs row_stride >= K, row_stride %% 8 == 0, batch_stride %% 8 == 0 and a 16-byte aligned base");
    hipError_t e = amx::launch_quantize_contig(f.scale, f.asymmetric != 0, f.group_size, xb, rows, K, row_stride, batch,
                                               batch_stride, tensor_pair, codes, scales, s);
    return e == hipSuccess ? AMX_OK : hip_fail(e, "quantize launch");
  }
  if (row_stride == 1 && k_stride >= rows) {
    if (!aligned(x, 2)) return fail(AMX_ERR_INVALID_ARG, "x must be 2-byte aligned");
    if (rows > kMaxStridedRows)
      return fail(AMX_ERR_INVALID_ARG, "rows = %lld exceeds the maximum %lld of the strided cast", (long long)rows,
                  (long long)kMaxStridedRows);
    hipError_t e = amx::launch_quantize_strided(f.scale, f.asymmetric != 0, f.group_size, xb, rows, K, k_stride, batch,
                                                batch_stride, tensor_pair, codes, scales, s);
    return e == hipSuccess ? AMX_OK : hip_fail(e, "strided quantize launch");
  }
  return fail(AMX_ERR_INVALID_ARG, "unsupported strides: need k_stride == 1, or row_stride == 1 with k_stride >= rows");
}

int dequantize_impl(amx_format_t f, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                    const float* tensor_pair, void* out, int32_t out_dtype, void* stream) {
  if (int rc = check_format(&f, true)) return rc;
  if (int rc = check_shape(f, rows, K)) return rc;
  if (!codes || !scales || !out) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (out_dtype != 0 && out_dtype != 1) return fail(AMX_ERR_INVALID_ARG, "out_dtype must be 0 (f32) or 1 (bf16)");
  if (!aligned(codes, 4) || !aligned(scales, 2) || !aligned(out, 16))
    return fail(AMX_ERR_INVALID_ARG, "misaligned pointer");
  hipError_t e = amx::launch_dequantize(f.scale, f.asymmetric != 0, f.group_size, codes, scales, rows, K, tensor_pair, out,
                                        out_dtype,
                                        reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AMX_OK : hip_fail(e, "dequantize launch");
}

// Power-of-two scales of 32-element groups go to the block-scaled matrix instructions (whose blocks are 32 long); FP8
// scales, other group sizes, and shapes those paths do not take, go through exact BF16 expansion.
bool uses_fp4_mfma(const amx_format_t& f, int64_t M, int64_t N, int64_t K) {
  return f.group_size == 32 && (f.scale == AMX_SCALE_E8M0_FLOOR || f.scale == AMX_SCALE_E8M0_ROUND) && amx::fp4_path_supported(M, N, K);
}

// A few rows on the A side (M <= 256; up to 768 for a single problem against a large B) with groups of 32: the
// weights-bound kernel that reads B's codes directly.
bool uses_skinny(const amx_format_t& f, int64_t M, int64_t N, int64_t K, int64_t batch) {
  return f.group_size == 32 && amx::skinny_path_supported(M, N, K, batch);
}

// What one GEMM call runs: resolved ONCE per call from the format, the shape and the caller's options, and used for
// both the workspace requirement and the dispatch (a kernel that does not take the shape falls back to the default).
enum GemmKernel : int { kGemmSkinny, kGemmFp8Merged, kGemmFp6Merged, kGemmFp4, kGemmE5m2Fused, kGemmE5m2Hybrid, kGemmPanel };
struct GemmPlan {
  GemmKernel kernel;
  int tile;           // BF16-panel kernel: AMX_TILE_*
  int skinny_slices;  // few-rows kernel: forced outer K slices, 0 = cost model
};

int check_options(const amx_gemm_options_t* o) {
  if (!o) return AMX_OK;
  if (o->e5m2_kernel < AMX_E5M2_PANEL || o->e5m2_kernel > AMX_E5M2_FUSED)
    return fail(AMX_ERR_INVALID_ARG, "options: no such e5m2_kernel %d", (int)o->e5m2_kernel);
  if (o->pot_kernel < AMX_POT_MERGED_FP6 || o->pot_kernel > AMX_POT_MERGED_FP8)
    return fail(AMX_ERR_INVALID_ARG, "options: no such pot_kernel %d", (int)o->pot_kernel);
  if (o->tile < AMX_TILE_AUTO || o->tile > AMX_TILE_64x256)
    return fail(AMX_ERR_INVALID_ARG, "options: no such tile %d", (int)o->tile);
  if (o->few_rows < -1 || o->few_rows > 16)
    return fail(AMX_ERR_INVALID_ARG, "options: few_rows must be -1, 0 or a slice count up to 16 (got %d)", (int)o->few_rows);
  return AMX_OK;
}

// scaled: the tensor-wise double scaling (Sec. 5.3), which only the BF16-panel kernel's epilogue applies.
GemmPlan plan_gemm(const amx_format_t& f, const amx_gemm_options_t* o, bool scaled, int64_t M, int64_t N, int64_t K,
                   int64_t batch) {
  static const amx_gemm_options_t kDefaults = {0, 0, 0, 0};
  const amx_gemm_options_t& opt = o ? *o : kDefaults;
  GemmPlan p = {kGemmPanel, opt.tile, opt.few_rows > 0 ? opt.few_rows : 0};
  if (scaled) return p;
  if (opt.few_rows >= 0 && uses_skinny(f, M, N, K, batch)) return p.kernel = kGemmSkinny, p;
  const bool pot32 = f.group_size == 32 && (f.scale == AMX_SCALE_E8M0_FLOOR || f.scale == AMX_SCALE_E8M0_ROUND);
  if (pot32 && f.asymmetric) {
    if (opt.pot_kernel == AMX_POT_SPLIT_FP4 && amx::fp4_path_supported(M, N, K)) return p.kernel = kGemmFp4, p;
    if (opt.pot_kernel != AMX_POT_MERGED_FP8 && amx::fp6m_path_supported(M, N, K)) return p.kernel = kGemmFp6Merged, p;
    return p.kernel = kGemmFp8Merged, p;
  }
  if (uses_fp4_mfma(f, M, N, K)) return p.kernel = kGemmFp4, p;
  if (f.scale == AMX_SCALE_FP8_E5M2 && f.group_size == 32) {
    if (opt.e5m2_kernel == AMX_E5M2_FUSED && amx::e5m2_fused_supported(M, N, K)) return p.kernel = kGemmE5m2Fused, p;
    if (opt.e5m2_kernel == AMX_E5M2_HYBRID && amx::e5m2_hybrid_supported(M, N, K)) return p.kernel = kGemmE5m2Hybrid, p;
  }
  return p;
}

size_t plan_workspace_bytes(const GemmPlan& p, bool asym, int64_t M, int64_t N, int64_t K, int64_t batch) {
  switch (p.kernel) {
    case kGemmSkinny: return amx::skinny_path_workspace_bytes(M, N, K, batch, p.skinny_slices);
    case kGemmFp8Merged: return amx::fp8m_path_workspace_bytes(M, N, K, batch);
    case kGemmFp6Merged: return amx::fp6m_path_workspace_bytes(M, N, K, batch);
    case kGemmFp4: return amx::fp4_path_workspace_bytes(asym, M, N, K, batch);
    case kGemmE5m2Fused: return 0;
    case kGemmE5m2Hybrid: return amx::e5m2_hybrid_workspace_bytes(M, K, batch);
    default: return amx::bf16_path_workspace_bytes(M, N, K, batch);
  }
}

// A_pair / B_pair: device {S_t, 1 / S_t} of the operands' tensor-wise scales (Sec. 5.3), both null for none. Scaled
// products always take the BF16 expansion path, whose kernel has the scaling epilogue.
int gemm_impl(amx_format_t f, const amx_gemm_options_t* opts, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
              const uint8_t* A_scales, const float* A_pair, const uint8_t* B_codes, const uint8_t* B_scales,
              const float* B_pair, float* C, int64_t ldc, int64_t batch, void* workspace, size_t workspace_bytes,
              void* stream, const void* B_panel = nullptr) {
  const bool scaled = A_pair != nullptr;
  if (int rc = check_format(&f, true)) return rc;
  if (int rc = check_options(opts)) return rc;
  if (int rc = check_shape(f, M, K)) return rc;
  if (N <= 0 || batch <= 0) return fail(AMX_ERR_INVALID_ARG, "N and batch must be positive");
  if (M > kMaxGemmRows || N > kMaxGemmRows || batch > kMaxBatch)
    return fail(AMX_ERR_INVALID_ARG, "M and N may be at most %lld and batch at most %lld (got %lld, %lld, %lld)",
                (long long)kMaxGemmRows, (long long)kMaxBatch, (long long)M, (long long)N, (long long)batch);
  if (ldc < N) return fail(AMX_ERR_INVALID_ARG, "ldc < N");
  if (ldc > kMaxLdc) return fail(AMX_ERR_INVALID_ARG, "ldc = %lld exceeds the supported maximum %lld", (long long)ldc, (long long)kMaxLdc);
  if (!A_codes || !A_scales || !B_codes || !B_scales || !C) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(A_codes, 16) || !aligned(B_codes, 16) || !aligned(A_scales, 4) || !aligned(B_scales, 4) ||
      !aligned(C, 4))
    return fail(AMX_ERR_INVALID_ARG, "codes need 16-byte, scales and C 4-byte alignment");
  const GemmPlan plan = plan_gemm(f, opts, scaled, M, N, K, batch);
  // a prepared B is read by the BF16-panel kernel (its expansion) and by the merged FP6 kernel (its own panel)
  if (plan.kernel != kGemmPanel && plan.kernel != kGemmFp6Merged) B_panel = nullptr;
  const size_t need = !B_panel ? plan_workspace_bytes(plan, f.asymmetric != 0, M, N, K, batch)
                      : plan.kernel == kGemmPanel ? amx::bf16_panel_bytes(M, K) : amx::fp6m_prepared_workspace_bytes(M, N, K);
  if (need > 0) {
    if (!workspace || workspace_bytes < need)
      return fail(AMX_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : 0);
    if (!aligned(workspace, 256)) return fail(AMX_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  }
  const amx::KernelTimer timer = g_timer;
  g_timer = amx::KernelTimer();
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  const bool asym = f.asymmetric != 0;
  hipError_t e;
  switch (plan.kernel) {
    case kGemmSkinny:
      e = amx::launch_gemm_skinny_path(f.scale, asym, M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch,
                                       workspace, plan.skinny_slices, hs, timer);
      break;
    case kGemmFp8Merged:
      e = amx::launch_gemm_fp8m_path(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace, hs, timer);
      break;
    case kGemmFp6Merged:
      e = B_panel ? amx::launch_gemm_fp6m_prepared(M, N, K, A_codes, A_scales, B_panel, C, ldc, workspace, hs, timer)
                  : amx::launch_gemm_fp6m_path(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace,
                                               hs, timer);
      break;
    case kGemmFp4:
      e = amx::launch_gemm_fp4_path(asym, M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace, hs,
                                    timer);
      break;
    case kGemmE5m2Fused:
      e = amx::launch_gemm_e5m2_fused(asym, M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, hs, timer);
      break;
    case kGemmE5m2Hybrid:
      e = amx::launch_gemm_e5m2_hybrid(asym, M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace,
                                       hs, timer);
      break;
    default:
      e = amx::launch_gemm_bf16_path(f.scale, asym, f.group_size, M, N, K, A_codes, A_scales, B_codes, B_scales, A_pair,
                                     B_pair, C, ldc, batch, workspace, plan.tile, hs, timer, false, B_panel);
  }
  return e == hipSuccess ? AMX_OK : hip_fail(e, "gemm launch");
}

// The gated GEMM runs on the tiled kernels only (the block-scaled ones for power-of-two scales, else the BF16 panels).
GemmPlan plan_glu(const amx_format_t& f, int64_t M, int64_t N, int64_t K) {
  static const amx_gemm_options_t kTiledOnly = {0, AMX_POT_MERGED_FP6, 0, -1};
  GemmPlan p = plan_gemm(f, &kTiledOnly, false, M, N, K, 1);
  if (p.kernel != kGemmFp6Merged && p.kernel != kGemmFp8Merged && p.kernel != kGemmFp4) p.kernel = kGemmPanel;
  return p;
}
size_t glu_workspace_bytes(const amx_format_t& f, int64_t M, int64_t N, int64_t K) {
  return plan_workspace_bytes(plan_glu(f, M, N, K), f.asymmetric != 0, M, N, K, 1);
}

amx_format_t symmetric(const amx_format_t* f) {
  amx_format_t g = *f;
  g.asymmetric = 0;
  return g;
}

}  // namespace

extern "C" {

const char* amxfp4_last_error(void) { return g_err; }

int amxfp4_profile_next_gemm(void* start_event, void* stop_event) {
  g_timer.start = reinterpret_cast<hipEvent_t>(start_event);
  g_timer.stop = reinterpret_cast<hipEvent_t>(stop_event);
  return AMX_OK;
}

size_t amxfp4_codes_bytes(const amx_format_t* fmt, int64_t rows, int64_t K) {
  if (!fmt || rows <= 0 || K <= 0 || K % 2) return 0;
  return (size_t)(rows * K / 2);
}

size_t amxfp4_scales_bytes(const amx_format_t* fmt, int64_t rows, int64_t K) {
  if (!fmt || rows <= 0 || K <= 0 || !amx::group_divides(K, fmt->group_size)) return 0;
  const int64_t groups = fmt->group_size == -1 ? 1 : K / fmt->group_size;
  return (size_t)(rows * groups * (fmt->asymmetric ? 2 : 1));
}

size_t amxfp4_gemm_workspace_bytes_ex(const amx_format_t* fmt, const amx_gemm_options_t* opts, int64_t M, int64_t N,
                                      int64_t K, int64_t batch) {
  if (!fmt || M <= 0 || N <= 0 || K <= 0 || batch <= 0 || check_options(opts)) return 0;
  return plan_workspace_bytes(plan_gemm(*fmt, opts, false, M, N, K, batch), fmt->asymmetric != 0, M, N, K, batch);
}

size_t amxfp4_gemm_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, int64_t batch) {
  return amxfp4_gemm_workspace_bytes_ex(fmt, nullptr, M, N, K, batch);
}

int amxfp4_quantize(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                    int64_t k_stride, uint8_t* codes, uint8_t* scales, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return quantize_impl(*fmt, x_bf16, 1, 0, rows, K, row_stride, k_stride, nullptr, codes, scales, stream);
}

int amxfp4_quantize_batched(const amx_format_t* fmt, const void* x_bf16, int64_t batch, int64_t batch_stride,
                            int64_t rows, int64_t K, int64_t row_stride, int64_t k_stride, uint8_t* codes,
                            uint8_t* scales, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return quantize_impl(*fmt, x_bf16, batch, batch_stride, rows, K, row_stride, k_stride, nullptr, codes, scales, stream);
}

size_t amxfp4_gemm_silu_mul_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K) {
  if (!fmt) return 0;
  amx_format_t f = *fmt;
  if (check_format(&f) || check_shape(f, M, K) || width <= 0 || width % 32 != 0 || 2 * width > kMaxGemmRows ||
      M > kMaxGemmRows)
    return 0;
  return glu_workspace_bytes(f, M, 2 * width, K);
}

int amxfp4_rmsnorm_quantize(const amx_format_t* fmt, const void* x_bf16, const float* y, void* sum_out_bf16,
                            const float* weight, int64_t rows, int64_t dim, float eps, uint8_t* codes, uint8_t* scales,
                            void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  amx_format_t f = *fmt;
  if (int rc = check_format(&f)) return rc;
  if (int rc = check_shape(f, rows, dim)) return rc;
  if (!amx::rmsnorm_quantize_supported(f.group_size, dim))
    return fail(AMX_ERR_UNSUPPORTED, "rmsnorm_quantize: groups of 16, 32 or 64 and dim <= 16384 only");
  if (rows > 0x7FFFFFFF) return fail(AMX_ERR_INVALID_ARG, "rmsnorm_quantize: too many rows");
  if (!x_bf16 || !weight || !codes || !scales) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if ((y != nullptr) != (sum_out_bf16 != nullptr))
    return fail(AMX_ERR_INVALID_ARG, "rmsnorm_quantize: y and sum_out_bf16 go together");
  if (!aligned(x_bf16, 16) || !aligned(weight, 16) || !aligned(codes, 16) || !aligned(scales, 4) ||
      (y && (!aligned(y, 16) || !aligned(sum_out_bf16, 16))))
    return fail(AMX_ERR_INVALID_ARG, "x, y, sum_out, weight and codes need 16-byte, scales 4-byte alignment");
  hipError_t e = amx::launch_rmsnorm_quantize(f.scale, f.asymmetric != 0, f.group_size,
                                              reinterpret_cast<const uint16_t*>(x_bf16), y,
                                              reinterpret_cast<uint16_t*>(sum_out_bf16), weight, rows, dim, eps, codes,
                                              scales, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AMX_OK : hip_fail(e, "rmsnorm_quantize launch");
}

// B_panel: the prepared form of the interleaved weights (amxfp4_prepare_weights on [2 * width][K]), or null
static int glu_impl(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K, const uint8_t* A_codes,
                    const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, const void* B_panel,
                    void* out_bf16, int64_t ld_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  amx_format_t f = *fmt;
  if (int rc = check_format(&f)) return rc;
  if (int rc = check_shape(f, M, K)) return rc;
  if (width <= 0 || width % 32 != 0) return fail(AMX_ERR_INVALID_ARG, "gemm_silu_mul: width must be a positive multiple of 32");
  if (M > kMaxGemmRows || 2 * width > kMaxGemmRows)
    return fail(AMX_ERR_INVALID_ARG, "gemm_silu_mul: M and 2 * width may be at most %lld", (long long)kMaxGemmRows);
  if (ld_out < width) return fail(AMX_ERR_INVALID_ARG, "gemm_silu_mul: ld_out < width");
  if (!A_codes || !A_scales || !B_codes || !B_scales || !out_bf16) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(A_codes, 16) || !aligned(B_codes, 16) || !aligned(A_scales, 4) || !aligned(B_scales, 4) ||
      !aligned(out_bf16, 2))
    return fail(AMX_ERR_INVALID_ARG, "codes need 16-byte, scales 4-byte, out 2-byte alignment");
  const GemmKernel glu_kernel = plan_glu(f, M, 2 * width, K).kernel;
  if (glu_kernel != kGemmPanel && glu_kernel != kGemmFp6Merged) B_panel = nullptr;
  const size_t need = !B_panel ? glu_workspace_bytes(f, M, 2 * width, K)
                      : glu_kernel == kGemmPanel ? amx::bf16_panel_bytes(M, K)
                                                 : amx::fp6m_prepared_workspace_bytes(M, 2 * width, K);
  if (need > 0) {
    if (!workspace || workspace_bytes < need)
      return fail(AMX_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : 0);
    if (!aligned(workspace, 256)) return fail(AMX_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  }
  const amx::KernelTimer timer = g_timer;
  g_timer = amx::KernelTimer();
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  float* out = reinterpret_cast<float*>(out_bf16);
  if (glu_kernel == kGemmFp8Merged) {
    hipError_t e = amx::launch_gemm_fp8m_path(M, 2 * width, K, A_codes, A_scales, B_codes, B_scales, out, ld_out, 1,
                                              workspace, hs, timer, true);
    return e == hipSuccess ? AMX_OK : hip_fail(e, "gemm_silu_mul launch");
  }
  if (glu_kernel == kGemmFp6Merged) {
    hipError_t e = B_panel ? amx::launch_gemm_fp6m_prepared(M, 2 * width, K, A_codes, A_scales, B_panel, out, ld_out,
                                                            workspace, hs, timer, true)
                           : amx::launch_gemm_fp6m_path(M, 2 * width, K, A_codes, A_scales, B_codes, B_scales, out,
                                                        ld_out, 1, workspace, hs, timer, true);
    return e == hipSuccess ? AMX_OK : hip_fail(e, "gemm_silu_mul launch");
  }
  if (glu_kernel == kGemmFp4) {
    hipError_t e = amx::launch_gemm_fp4_path(f.asymmetric != 0, M, 2 * width, K, A_codes, A_scales, B_codes, B_scales,
                                             out, ld_out, 1, workspace, hs, timer, true);
    return e == hipSuccess ? AMX_OK : hip_fail(e, "gemm_silu_mul launch");
  }
  hipError_t e = amx::launch_gemm_bf16_path(f.scale, f.asymmetric != 0, f.group_size, M, 2 * width, K, A_codes, A_scales,
                                            B_codes, B_scales, nullptr, nullptr, reinterpret_cast<float*>(out_bf16),
                                            ld_out, 1, workspace, AMX_TILE_AUTO, reinterpret_cast<hipStream_t>(stream), timer,
                                            true, B_panel);
  return e == hipSuccess ? AMX_OK : hip_fail(e, "gemm_silu_mul launch");
}

int amxfp4_gemm_silu_mul(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K, const uint8_t* A_codes,
                         const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, void* out_bf16,
                         int64_t ld_out, void* workspace, size_t workspace_bytes, void* stream) {
  return glu_impl(fmt, M, width, K, A_codes, A_scales, B_codes, B_scales, nullptr, out_bf16, ld_out, workspace,
                  workspace_bytes, stream);
}

size_t amxfp4_gemm_silu_mul_prepared_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K) {
  const size_t plain = amxfp4_gemm_silu_mul_workspace_bytes(fmt, M, width, K);
  if (plain == 0 || amxfp4_weights_prepared_bytes(fmt, 2 * width, K) == 0) return plain;
  const GemmKernel kernel = plan_glu(*fmt, M, 2 * width, K).kernel;
  return kernel == kGemmPanel        ? amx::bf16_panel_bytes(M, K)
         : kernel == kGemmFp6Merged ? amx::fp6m_prepared_workspace_bytes(M, 2 * width, K)
                                    : plain;
}

int amxfp4_gemm_silu_mul_prepared(const amx_format_t* fmt, int64_t M, int64_t width, int64_t K, const uint8_t* A_codes,
                                  const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales,
                                  const void* prepared, size_t prepared_bytes, void* out_bf16, int64_t ld_out,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  const size_t need = width > 0 && K > 0 ? amxfp4_weights_prepared_bytes(fmt, 2 * width, K) : 0;
  if (need > 0) {
    if (!prepared || prepared_bytes < need)
      return fail(AMX_ERR_WORKSPACE, "prepared buffer of %zu bytes needed, %zu given", need, prepared ? prepared_bytes : 0);
    if (!aligned(prepared, 256)) return fail(AMX_ERR_INVALID_ARG, "prepared buffer must be 256-byte aligned");
  }
  return glu_impl(fmt, M, width, K, A_codes, A_scales, B_codes, B_scales, need > 0 ? prepared : nullptr, out_bf16, ld_out,
                  workspace, workspace_bytes, stream);
}

int amxfp4_dequantize(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                      void* out, int32_t out_dtype, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return dequantize_impl(*fmt, codes, scales, rows, K, nullptr, out, out_dtype, stream);
}

int amxfp4_gemm(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                int64_t batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return gemm_impl(*fmt, nullptr, M, N, K, A_codes, A_scales, nullptr, B_codes, B_scales, nullptr, C, ldc, batch, workspace,
                   workspace_bytes, stream);
}

int amxfp4_gemm_ex(const amx_format_t* fmt, const amx_gemm_options_t* opts, int64_t M, int64_t N, int64_t K,
                   const uint8_t* A_codes, const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales,
                   float* C, int64_t ldc, int64_t batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return gemm_impl(*fmt, opts, M, N, K, A_codes, A_scales, nullptr, B_codes, B_scales, nullptr, C, ldc, batch, workspace,
                   workspace_bytes, stream);
}

// Prepared weights: the formats whose large products run on the BF16-panel kernel have B's panel expanded once; the
// asymmetric power-of-two format has B's merged FP6 panel, anchors and plan written once; the symmetric power-of-two
// format's kernel reads the codes as they are.
size_t amxfp4_weights_prepared_bytes(const amx_format_t* fmt, int64_t N, int64_t K) {
  if (!fmt || N <= 0 || K <= 0 || check_format(fmt, true) != AMX_OK || !amx::group_divides(K, fmt->group_size)) return 0;
  const bool pot32 = fmt->group_size == 32 && (fmt->scale == AMX_SCALE_E8M0_FLOOR || fmt->scale == AMX_SCALE_E8M0_ROUND);
  if (!pot32) return amx::bf16_panel_bytes(N, K);
  return fmt->asymmetric && amx::fp6m_path_supported(1, N, K) ? amx::fp6m_prepared_bytes(N, K) : 0;
}

int amxfp4_prepare_weights(const amx_format_t* fmt, int64_t N, int64_t K, const uint8_t* B_codes,
                           const uint8_t* B_scales, void* prepared, size_t prepared_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (int rc = check_format(fmt, true)) return rc;
  if (int rc = check_shape(*fmt, N, K)) return rc;
  if (N > kMaxGemmRows) return fail(AMX_ERR_INVALID_ARG, "N may be at most %lld", (long long)kMaxGemmRows);
  if (!B_codes || !B_scales) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(B_codes, 16) || !aligned(B_scales, 4)) return fail(AMX_ERR_INVALID_ARG, "codes need 16-byte, scales 4-byte alignment");
  const size_t need = amxfp4_weights_prepared_bytes(fmt, N, K);
  if (need == 0) return AMX_OK;  // this format's kernels read B as it is stored
  if (!prepared || prepared_bytes < need)
    return fail(AMX_ERR_WORKSPACE, "prepared buffer of %zu bytes needed, %zu given", need, prepared ? prepared_bytes : 0);
  if (!aligned(prepared, 256)) return fail(AMX_ERR_INVALID_ARG, "prepared buffer must be 256-byte aligned");
  const bool pot32 = fmt->group_size == 32 && (fmt->scale == AMX_SCALE_E8M0_FLOOR || fmt->scale == AMX_SCALE_E8M0_ROUND);
  const hipError_t e =
      pot32 ? amx::launch_fp6m_prepare_b(N, K, B_codes, B_scales, prepared, reinterpret_cast<hipStream_t>(stream))
            : amx::launch_expand_b_panel(fmt->scale, fmt->asymmetric != 0, fmt->group_size, N, K, B_codes, B_scales,
                                         prepared, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AMX_OK : hip_fail(e, "prepare_weights launch");
}

size_t amxfp4_gemm_prepared_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K) {
  if (!fmt || M <= 0 || N <= 0 || K <= 0) return 0;
  const GemmPlan plan = plan_gemm(*fmt, nullptr, false, M, N, K, 1);
  if (amxfp4_weights_prepared_bytes(fmt, N, K) > 0) {
    if (plan.kernel == kGemmPanel) return amx::bf16_panel_bytes(M, K);
    if (plan.kernel == kGemmFp6Merged) return amx::fp6m_prepared_workspace_bytes(M, N, K);
  }
  return plan_workspace_bytes(plan, fmt->asymmetric != 0, M, N, K, 1);
}

int amxfp4_gemm_prepared(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                         const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, const void* prepared,
                         size_t prepared_bytes, float* C, int64_t ldc, void* workspace, size_t workspace_bytes,
                         void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (int rc = check_format(fmt, true)) return rc;
  const size_t need = N > 0 && K > 0 ? amxfp4_weights_prepared_bytes(fmt, N, K) : 0;
  if (need > 0) {
    if (!prepared || prepared_bytes < need)
      return fail(AMX_ERR_WORKSPACE, "prepared buffer of %zu bytes needed, %zu given", need, prepared ? prepared_bytes : 0);
    if (!aligned(prepared, 256)) return fail(AMX_ERR_INVALID_ARG, "prepared buffer must be 256-byte aligned");
  }
  return gemm_impl(*fmt, nullptr, M, N, K, A_codes, A_scales, nullptr, B_codes, B_scales, nullptr, C, ldc, 1, workspace,
                   workspace_bytes, stream, need > 0 ? prepared : nullptr);
}

int amxfp4_gemm_static(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                       const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
                       int64_t batch, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  // the size check comes first, on the host, from the same plan amxfp4_gemm would follow
  if (int rc = check_format(fmt, true)) return rc;
  if (int rc = check_shape(*fmt, M, K)) return rc;
  if (N <= 0 || batch <= 0 || M > kMaxGemmRows || N > kMaxGemmRows || batch > kMaxBatch)
    return fail(AMX_ERR_INVALID_ARG, "N and batch must be positive and M, N, batch within the limits of amxfp4_gemm");
  const size_t need = plan_workspace_bytes(plan_gemm(*fmt, nullptr, false, M, N, K, batch), fmt->asymmetric != 0, M, N, K, batch);
  if (need > kStaticScratchBytes)
    return fail(AMX_ERR_WORKSPACE, "this product needs %zu bytes of scratch; the static array holds %zu (use amxfp4_gemm "
                "with a workspace)", need, kStaticScratchBytes);
  void* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  return gemm_impl(*fmt, nullptr, M, N, K, A_codes, A_scales, nullptr, B_codes, B_scales, nullptr, C, ldc, batch, ptr,
                   kStaticScratchBytes, stream);
}

int mxfp4_quantize(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                   int64_t k_stride, uint8_t* codes, uint8_t* scales, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return quantize_impl(symmetric(fmt), x_bf16, 1, 0, rows, K, row_stride, k_stride, nullptr, codes, scales, stream);
}

int mxfp4_dequantize(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                     void* out, int32_t out_dtype, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return dequantize_impl(symmetric(fmt), codes, scales, rows, K, nullptr, out, out_dtype, stream);
}

int mxfp4_gemm(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
               const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc,
               int64_t batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  return gemm_impl(symmetric(fmt), nullptr, M, N, K, A_codes, A_scales, nullptr, B_codes, B_scales, nullptr, C, ldc,
                   batch, workspace, workspace_bytes, stream);
}

int amxfp4_tensor_scale(const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride, float* scale_pair,
                        void* stream) {
  if (!x_bf16 || !scale_pair) return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (rows <= 0 || K <= 0 || K % 8 != 0) return fail(AMX_ERR_INVALID_ARG, "rows and K must be positive, K a multiple of 8");
  if (row_stride < K || row_stride % 8 != 0 || !aligned(x_bf16, 16) || !aligned(scale_pair, 8))
    return fail(AMX_ERR_INVALID_ARG, "need row_stride >= K, row_stride %% 8 == 0, a 16-byte aligned tensor and an 8-byte aligned pair");
  hipError_t e = amx::launch_tensor_scale(reinterpret_cast<const uint16_t*>(x_bf16), rows, K, row_stride, scale_pair,
                                          reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AMX_OK : hip_fail(e, "tensor scale launch");
}

int amxfp4_quantize_scaled(const amx_format_t* fmt, const void* x_bf16, int64_t rows, int64_t K, int64_t row_stride,
                           int64_t k_stride, const float* scale_pair, uint8_t* codes, uint8_t* scales, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (!scale_pair || !aligned(scale_pair, 8)) return fail(AMX_ERR_INVALID_ARG, "scale_pair is NULL or misaligned");
  return quantize_impl(*fmt, x_bf16, 1, 0, rows, K, row_stride, k_stride, scale_pair, codes, scales, stream);
}

int amxfp4_dequantize_scaled(const amx_format_t* fmt, const uint8_t* codes, const uint8_t* scales, int64_t rows,
                             int64_t K, const float* scale_pair, float* out, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (!scale_pair || !aligned(scale_pair, 8)) return fail(AMX_ERR_INVALID_ARG, "scale_pair is NULL or misaligned");
  return dequantize_impl(*fmt, codes, scales, rows, K, scale_pair, out, 0, stream);
}

size_t amxfp4_gemm_scaled_workspace_bytes(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, int64_t batch) {
  if (!fmt || M <= 0 || N <= 0 || K <= 0 || batch <= 0) return 0;
  return amx::bf16_path_workspace_bytes(M, N, K, batch);
}

int amxfp4_gemm_scaled(const amx_format_t* fmt, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                       const uint8_t* A_scales, const float* A_scale_pair, const uint8_t* B_codes,
                       const uint8_t* B_scales, const float* B_scale_pair, float* C, int64_t ldc, int64_t batch,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (!A_scale_pair || !B_scale_pair || !aligned(A_scale_pair, 8) || !aligned(B_scale_pair, 8))
    return fail(AMX_ERR_INVALID_ARG, "a scale pair is NULL or misaligned");
  return gemm_impl(*fmt, nullptr, M, N, K, A_codes, A_scales, A_scale_pair, B_codes, B_scales, B_scale_pair, C, ldc,
                   batch, workspace, workspace_bytes, stream);
}

size_t amxfp4_attention_workspace_bytes(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq,
                                        int64_t Sk, int64_t head_dim) {
  if (!fmt || q_heads <= 0 || kv_heads <= 0 || Sq <= 0 || Sk <= 0 || (head_dim != 128 && head_dim != 64)) return 0;
  return amx::attention_workspace_bytes(q_heads, kv_heads, Sq, Sk, head_dim);
}

static int attention_impl(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                     int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                     const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                     int32_t causal, void* out, bool merged_bf16, void* workspace, size_t workspace_bytes,
                          void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (int rc = check_format(fmt)) return rc;
  if (fmt->group_size != 32) return fail(AMX_ERR_UNSUPPORTED, "the fused attention takes groups of 32 (one group per key tile)");
  if (head_dim != 128 && head_dim != 64)
    return fail(AMX_ERR_UNSUPPORTED, "the fused attention is built for head_dim 128 and 64 (got %lld)", (long long)head_dim);
  if (q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads != 0 || q_heads > 65535)
    return fail(AMX_ERR_INVALID_ARG, "q_heads must be a positive multiple of kv_heads (at most 65535)");
  if (Sq <= 0 || Sk <= 0 || Sk % 32 != 0 || Sk > (1 << 20) || Sq > (1 << 20))
    return fail(AMX_ERR_INVALID_ARG, "Sq and Sk must be positive, at most 2^20, and Sk a multiple of 32");
  if (causal != 0 && causal != 1) return fail(AMX_ERR_INVALID_ARG, "causal must be 0 or 1");
  if (causal && Sk < Sq) return fail(AMX_ERR_INVALID_ARG, "causal attention needs Sk >= Sq (queries are aligned to the end of the keys)");
  if (!(scale > 0.0f) || !(scale < 1.0e30f)) return fail(AMX_ERR_INVALID_ARG, "scale must be a positive finite number");
  if (!Q_codes || !Q_scales || !K_codes || !K_scales || !V_codes || !V_scales || !out)
    return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(Q_codes, 16) || !aligned(K_codes, 16) || !aligned(V_codes, 16) || !aligned(Q_scales, 2) ||
      !aligned(K_scales, 2) || !aligned(V_scales, 2) || !aligned(out, 16))
    return fail(AMX_ERR_INVALID_ARG, "codes and out need 16-byte, scales 2-byte alignment");
  const size_t need = amx::attention_workspace_bytes(q_heads, kv_heads, Sq, Sk, head_dim);
  if (!workspace || workspace_bytes < need)
    return fail(AMX_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : 0);
  if (!aligned(workspace, 256)) return fail(AMX_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  const amx::KernelTimer timer = g_timer;
  g_timer = amx::KernelTimer();
  hipError_t e = amx::launch_attention_fused(fmt->scale, fmt->asymmetric != 0, q_heads, kv_heads, Sq, Sk, head_dim, Q_codes,
                                             Q_scales, K_codes, K_scales, V_codes, V_scales, scale, causal,
                                             reinterpret_cast<float*>(out), merged_bf16, workspace, reinterpret_cast<hipStream_t>(stream), timer);
  return e == hipSuccess ? AMX_OK : hip_fail(e, "attention launch");
}

size_t amxfp4_attention_decode_workspace_bytes(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq,
                                               int64_t Sk, int64_t head_dim, int64_t key_splits) {
  if (!fmt || Sk <= 0 || key_splits <= 0 || !amx::attention_decode_supported(q_heads, kv_heads, Sq, head_dim)) return 0;
  return amx::attention_decode_workspace_bytes(kv_heads, head_dim, key_splits);
}

int amxfp4_attention_decode(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                            int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                            const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                            int32_t causal, int64_t key_splits, float* out, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (!fmt) return fail(AMX_ERR_INVALID_ARG, "fmt is NULL");
  if (int rc = check_format(fmt)) return rc;
  if (fmt->group_size != 32) return fail(AMX_ERR_UNSUPPORTED, "the fused attention takes groups of 32 (one group per key tile)");
  if (head_dim != 128 && head_dim != 64)
    return fail(AMX_ERR_UNSUPPORTED, "the fused attention is built for head_dim 128 and 64 (got %lld)", (long long)head_dim);
  if (q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads != 0 || kv_heads > 65535)
    return fail(AMX_ERR_INVALID_ARG, "q_heads must be a positive multiple of kv_heads (kv_heads at most 65535)");
  if (Sq <= 0 || Sk <= 0 || Sk % 32 != 0 || Sk > (1 << 20))
    return fail(AMX_ERR_INVALID_ARG, "Sq and Sk must be positive, Sk a multiple of 32 and at most 2^20");
  if ((q_heads / kv_heads) * Sq > 32)
    return fail(AMX_ERR_UNSUPPORTED, "attention_decode takes at most 32 queries per key/value head ((q_heads / kv_heads) * Sq = "
                "%lld); use amxfp4_attention", (long long)((q_heads / kv_heads) * Sq));
  if (key_splits <= 0 || key_splits > 1024 || key_splits > Sk / 32)
    return fail(AMX_ERR_INVALID_ARG, "key_splits must be between 1 and min(1024, Sk / 32)");
  if (causal != 0 && causal != 1) return fail(AMX_ERR_INVALID_ARG, "causal must be 0 or 1");
  if (causal && Sk < Sq) return fail(AMX_ERR_INVALID_ARG, "causal attention needs Sk >= Sq (queries are aligned to the end of the keys)");
  if (!(scale > 0.0f) || !(scale < 1.0e30f)) return fail(AMX_ERR_INVALID_ARG, "scale must be a positive finite number");
  if (!Q_codes || !Q_scales || !K_codes || !K_scales || !V_codes || !V_scales || !out)
    return fail(AMX_ERR_INVALID_ARG, "NULL data pointer");
  if (!aligned(Q_codes, 16) || !aligned(K_codes, 16) || !aligned(V_codes, 16) || !aligned(Q_scales, 2) ||
      !aligned(K_scales, 2) || !aligned(V_scales, 2) || !aligned(out, 16))
    return fail(AMX_ERR_INVALID_ARG, "codes and out need 16-byte, scales 2-byte alignment");
  const size_t need = amx::attention_decode_workspace_bytes(kv_heads, head_dim, key_splits);
  if (!workspace || workspace_bytes < need)
    return fail(AMX_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : 0);
  if (!aligned(workspace, 256)) return fail(AMX_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  hipError_t e = amx::launch_attention_decode(fmt->scale, fmt->asymmetric != 0, q_heads, kv_heads, Sq, Sk, head_dim, Q_codes,
                                              Q_scales, K_codes, K_scales, V_codes, V_scales, scale, causal,
                                              (int)key_splits, out, workspace, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AMX_OK : hip_fail(e, "attention_decode launch");
}

int amxfp4_attention(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                     int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                     const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                     int32_t causal, float* out, void* workspace, size_t workspace_bytes, void* stream) {
  return attention_impl(fmt, q_heads, kv_heads, Sq, Sk, head_dim, Q_codes, Q_scales, K_codes, K_scales, V_codes,
                        V_scales, scale, causal, out, false, workspace, workspace_bytes, stream);
}

int amxfp4_attention_merged(const amx_format_t* fmt, int64_t q_heads, int64_t kv_heads, int64_t Sq, int64_t Sk,
                            int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                            const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                            int32_t causal, void* out_bf16, void* workspace, size_t workspace_bytes, void* stream) {
  return attention_impl(fmt, q_heads, kv_heads, Sq, Sk, head_dim, Q_codes, Q_scales, K_codes, K_scales, V_codes,
                        V_scales, scale, causal, out_bf16, true, workspace, workspace_bytes, stream);
}

}  // extern "C"
