// Fully quantized GEMM (Sec. 4.3) for a small number of rows on the A side (M <= 256: a few tokens against a weight
// matrix). Such a product is bound by reading the weights, and the point of 4-bit weights is that they are a quarter
// of the BF16 bytes, so this kernel reads the packed codes and scales of B straight from memory, dequantizes them in
// registers to exact BF16 (element * scale has at most 6 significant bits) and feeds the BF16 MFMA; only the small
// A operand goes through a BF16 panel (expand_kernel). No operand of B is ever written back.
//
// Work split: one workgroup = 4 waves = 4 neighbouring tiles of 32 columns of C (32 rows of B each) over one outer K
// slice. K is walked in blocks of 256. The workgroup brings the A operand into LDS once, by direct-to-LDS loads, in
// half blocks (M x 128 BF16 = 8 fragments per 32 rows), double buffered; each lane owns one B row (lane % 32 of its wave's
// tile) and loads that row's 128 bytes of codes (one cache line, fetched exactly once) and its 8 scale entries one
// block ahead, then runs 16 k-steps of 16 from registers: lane half h = lane / 32 turns codes 16 j + 8 h .. + 7 of a
// group into the 8 BF16 of its B fragment. With more than one outer slice the partial tiles go to the workspace and a
// second kernel adds them in a fixed order (no atomics: results are reproducible).
#include <stdlib.h>

#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// scale arrays are only 4-byte aligned by contract: vectors of them are loaded through under-aligned types
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));

typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two FP4 codes (byte SEL of `word`) -> their dequantized values as a pair of BF16: the hardware FP4 -> FP32
// conversion gives the signed elements, each is multiplied by the scale of its sign class (picked with the sign bit
// smeared over the word) and the product, which has at most 6 significant bits, is truncated to BF16 exactly.
template <bool ASYM, int SEL>
__device__ __forceinline__ uint32_t dequant2(uint32_t word, float s_pos, float s_neg) {
  const f32x2 e = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, SEL);
  float v0, v1;
  if constexpr (ASYM) {
    const uint32_t m0 = (uint32_t)((int32_t)f2u(e[0]) >> 31), m1 = (uint32_t)((int32_t)f2u(e[1]) >> 31);
    v0 = e[0] * u2f((f2u(s_neg) & m0) | (f2u(s_pos) & ~m0));
    v1 = e[1] * u2f((f2u(s_neg) & m1) | (f2u(s_pos) & ~m1));
  } else {
    v0 = e[0] * s_pos;
    v1 = e[1] * s_pos;
  }
  return __builtin_amdgcn_perm(f2u(v1), f2u(v0), 0x07060302u);  // upper halves: (v0 low, v1 high)
}

constexpr int kSkinnyMaxM = 256;    // at most eight 32-row MFMA tiles
constexpr int kSkinnyBlockK = 256;  // K block: 128 bytes of codes per row

// Outer K slices for a problem with `groups` workgroups per slice and nblk K blocks: about 512 workgroups (two per CU,
// 4 waves each) if the K blocks allow it. Returns the number of slices and sets the blocks per slice; every slice has
// at least one block ((slices - 1) * blocks_per_slice < nblk).
static int skinny_outer_slices(int64_t groups, int64_t nblk, int& blocks_per_slice) {
  int64_t want = (512 + groups - 1) / groups;
  want = want < 1 ? 1 : (want > nblk ? nblk : want);
  blocks_per_slice = (int)((nblk + want - 1) / want);
  return (int)((nblk + blocks_per_slice - 1) / blocks_per_slice);
}

// 32-row tiles the kernel is instantiated for: 1 .. 4, 6, 8 (A's panel and the partial tiles are padded to that)
static int skinny_row_tiles(int64_t M) {
  const int t = (int)((M + 31) / 32);
  return t <= 4 ? t : (t <= 6 ? 6 : 8);
}

bool skinny_path_supported(int64_t M, int64_t N, int64_t K) {
  static const bool enabled = !(getenv("AMXFP4_SKINNY") && atoi(getenv("AMXFP4_SKINNY")) == 0);
  return enabled && M <= kSkinnyMaxM && K % kSkinnyBlockK == 0 && N >= 1;
}

size_t skinny_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch) {
  const int64_t Mp = 32 * skinny_row_tiles(M);
  int bps;
  const int slices = skinny_outer_slices((N + 127) / 128 * batch, K / kSkinnyBlockK, bps);
  size_t bytes = (size_t)(batch * Mp * K * 2);                         // A panel
  bytes = (bytes + 255) / 256 * 256;
  if (slices > 1) bytes += (size_t)(batch * slices * Mp * N * 4);      // partial tiles
  return bytes;
}

// grid: (ceil(N / 128), outer slices, batch); block 256 = 4 waves.
// out: C (ld_out = ldc) when gridDim.y == 1, else partials [batch][slice][MT * 32][N].
template <int SCALE_KIND, bool ASYM, int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const uint16_t* __restrict__ Ap,
                                                          const uint8_t* __restrict__ B_codes,
                                                          const uint8_t* __restrict__ B_scales, float* __restrict__ out,
                                                          int64_t M, int64_t N, int64_t K, int64_t ld_out,
                                                          int64_t batch_stride_out, int64_t slice_stride_out,
                                                          int blocks_per_slice) {
  constexpr int kFragsPerHalf = MT * (kSkinnyBlockK / 32);  // A fragments of half a K block (8 k-steps)
  // two stages, separate arrays so that loads into one are known not to alias reads of the other
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kFragsPerHalf * kFragBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kFragsPerHalf * kFragBytes];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = lane >> 5;
  const int64_t b = blockIdx.z;
  const int64_t n = ((int64_t)blockIdx.x * 4 + wave) * 32 + (lane & 31);
  const bool valid = n < N;
  const int64_t G = K >> 5, nblk = K / kSkinnyBlockK;
  constexpr int kScaleBytes = ASYM ? 2 : 1;

  const int64_t s_begin = (int64_t)blockIdx.y * blocks_per_slice;
  const int nb = (int)((s_begin + blocks_per_slice < nblk ? s_begin + blocks_per_slice : nblk) - s_begin);  // >= 1

  const int64_t row = valid ? b * N + n : 0;  // (rows past N read row 0 and are discarded)
  const uint8_t* codes_row = B_codes + row * (K >> 1) + s_begin * (kSkinnyBlockK / 2);
  const uint8_t* scales_row = B_scales + (row * G + s_begin * 8) * kScaleBytes;
  // A panel of this batch entry: [MT row blocks][K / 16 fragments][64 lanes][8 BF16]; raw buffer, reads past the end
  // return zero
  const int kfrags = (int)(K >> 4);
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(Ap) + b * (int64_t)MT * kfrags * kFragBytes), 0,
      MT * kfrags * kFragBytes, 0x00020000);
  const int lane_off = lane * 16;
  const int first_frag = (int)s_begin * (kSkinnyBlockK / 16);

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;

  // wave w brings fragments w, w + 4, .. of A half block HB (of this slice) into stage DST: fragment f = row block
  // f / 8, k-step f % 8 of the half
#define AMX_SKINNY_LOAD_A(HB, DST)                                                                                 \
  _Pragma("unroll") for (int i_ = 0; i_ < kFragsPerHalf / 4; ++i_) {                                               \
    const int f_ = wave + 4 * i_;                                                                                  \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,               \
                                             ((f_ >> 3) * kfrags + first_frag + (HB) * 8 + (f_ & 7)) * kFragBytes,  \
                                             0, 0);                                                                \
  }
  // this lane's row: one cache line of codes (8 groups) and the 8 scale entries of block I
#define AMX_SKINNY_LOAD_B(I, W, S)                                                                                 \
  {                                                                                                                \
    const u32x4* csrc_ = reinterpret_cast<const u32x4*>(codes_row + (int64_t)(I) * (kSkinnyBlockK / 2));           \
    W[0] = csrc_[0], W[1] = csrc_[1], W[2] = csrc_[2], W[3] = csrc_[3];                                            \
    W[4] = csrc_[4], W[5] = csrc_[5], W[6] = csrc_[6], W[7] = csrc_[7];                                            \
    if constexpr (ASYM) {                                                                                          \
      const u32x4_a4 t_ = *reinterpret_cast<const u32x4_a4*>(scales_row + (int64_t)(I) * 16);                      \
      S[0] = t_[0], S[1] = t_[1], S[2] = t_[2], S[3] = t_[3];                                                      \
    } else {                                                                                                       \
      const u32x2_a4 t_ = *reinterpret_cast<const u32x2_a4*>(scales_row + (int64_t)(I) * 8);                       \
      S[0] = t_[0], S[1] = t_[1], S[2] = 0, S[3] = 0;                                                              \
    }                                                                                                              \
  }
  // The two k-steps of group GI (a literal: register arrays must not be indexed with a run-time value) of one block:
  // A fragments from stage SRC (the half block that holds the group), B from the registers W / S
#define AMX_SKINNY_GROUP(SRC, W, S, GI)                                                                            \
  {                                                                                                                \
    float s_pos, s_neg;                                                                                            \
    if constexpr (ASYM) {                                                                                          \
      const uint32_t sb = (S[(GI) >> 1] >> (16 * ((GI) & 1))) & 0xFFFFu;                                           \
      s_pos = scale_value<SCALE_KIND>(sb & 255u);                                                                  \
      s_neg = scale_value<SCALE_KIND>(sb >> 8);                                                                    \
    } else {                                                                                                       \
      const uint32_t sb = (S[(GI) >> 2] >> (8 * ((GI) & 3))) & 255u;                                               \
      s_pos = s_neg = scale_value<SCALE_KIND>(sb);                                                                 \
    }                                                                                                              \
    /* codes 16 j + 8 h .. + 7 of the group are word 2 j + h of its four */                                        \
    const uint32_t word0 = h ? W[GI][1] : W[GI][0], word1 = h ? W[GI][3] : W[GI][2];                               \
    const bf16x8 b0 = __builtin_bit_cast(bf16x8, u32x4{dequant2<ASYM, 0>(word0, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 1>(word0, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 2>(word0, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 3>(word0, s_pos, s_neg)});                   \
    const bf16x8 b1 = __builtin_bit_cast(bf16x8, u32x4{dequant2<ASYM, 0>(word1, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 1>(word1, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 2>(word1, s_pos, s_neg),                     \
                                                       dequant2<ASYM, 3>(word1, s_pos, s_neg)});                   \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                                            \
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>((SRC) + (mt * 8 + ((GI) & 3) * 2) * kFragBytes + lane_off); \
      const bf16x8 a1 =                                                                                            \
          *reinterpret_cast<const bf16x8*>((SRC) + (mt * 8 + ((GI) & 3) * 2 + 1) * kFragBytes + lane_off);         \
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[mt], 0, 0, 0);                                 \
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[mt], 0, 0, 0);                                 \
    }                                                                                                              \
  }
#define AMX_SKINNY_HALF0(SRC, W, S)                                                                                \
  AMX_SKINNY_GROUP(SRC, W, S, 0) AMX_SKINNY_GROUP(SRC, W, S, 1) AMX_SKINNY_GROUP(SRC, W, S, 2)                     \
  AMX_SKINNY_GROUP(SRC, W, S, 3)
#define AMX_SKINNY_HALF1(SRC, W, S)                                                                                \
  AMX_SKINNY_GROUP(SRC, W, S, 4) AMX_SKINNY_GROUP(SRC, W, S, 5) AMX_SKINNY_GROUP(SRC, W, S, 6)                     \
  AMX_SKINNY_GROUP(SRC, W, S, 7)

  u32x4 w0[8], w1[8];
  uint32_t s0[4], s1[4];
  AMX_SKINNY_LOAD_A(0, ldsA0);
  AMX_SKINNY_LOAD_B(0, w0, s0);
  AMX_WAIT_VMCNT(0);
  AMX_BARRIER();
  // Block i: its first half is multiplied from stage 0, its second from stage 1, with the codes in register set
  // i % 2. Every step fetches what the next step needs (the other A stage; the next block's codes during a first half)
  // and ends with a wait and a barrier, after which the stage it read may be refilled. All conditions are uniform.
  for (int i = 0; i < nb; i += 2) {
    AMX_SKINNY_LOAD_A(2 * i + 1, ldsA1);
    if (i + 1 < nb) AMX_SKINNY_LOAD_B(i + 1, w1, s1);
    AMX_SKINNY_HALF0(ldsA0, w0, s0);
    AMX_WAIT_VMCNT(0);
    AMX_BARRIER();
    if (i + 1 < nb) AMX_SKINNY_LOAD_A(2 * i + 2, ldsA0);
    AMX_SKINNY_HALF1(ldsA1, w0, s0);
    AMX_WAIT_VMCNT(0);
    AMX_BARRIER();
    if (i + 1 < nb) {
      AMX_SKINNY_LOAD_A(2 * i + 3, ldsA1);
      if (i + 2 < nb) AMX_SKINNY_LOAD_B(i + 2, w0, s0);
      AMX_SKINNY_HALF0(ldsA0, w1, s1);
      AMX_WAIT_VMCNT(0);
      AMX_BARRIER();
      if (i + 2 < nb) AMX_SKINNY_LOAD_A(2 * i + 4, ldsA0);
      AMX_SKINNY_HALF1(ldsA1, w1, s1);
      AMX_WAIT_VMCNT(0);
      AMX_BARRIER();
    }
  }
#undef AMX_SKINNY_HALF1
#undef AMX_SKINNY_HALF0
#undef AMX_SKINNY_GROUP
#undef AMX_SKINNY_LOAD_B
#undef AMX_SKINNY_LOAD_A

  // register v of row tile mt is row 32 mt + 8 (v / 4) + 4 h + v % 4, column n
  if (!valid) return;
  float* dst = out + b * batch_stride_out + (int64_t)blockIdx.y * slice_stride_out + n;
  const int64_t row_limit = gridDim.y == 1 ? M : (int64_t)MT * 32;  // partial tiles keep their padded rows
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t r = mt * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
      if (r < row_limit) dst[r * ld_out] = acc[mt][v];
    }
}

// C[b][r][c] = sum over slices of partial[b][slice][r][c], slices added in ascending order
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const float* __restrict__ partial, float* __restrict__ C,
                                                            int64_t M, int64_t N, int64_t Mp, int64_t ldc, int slices) {
  const int64_t b = blockIdx.z;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * N) return;
  const int64_t r = idx / N, c = idx - r * N;
  const float* p = partial + (b * slices * Mp + r) * N + c;
  float s = p[0];
  for (int k = 1; k < slices; ++k) s += p[(int64_t)k * Mp * N];
  C[(b * M + r) * ldc + c] = s;
}

template <int SK, bool ASYM, int MT>
static hipError_t launch_skinny(const uint16_t* Ap, const uint8_t* Bc, const uint8_t* Bs, float* C, float* partial,
                                int64_t M, int64_t N, int64_t K, int64_t ldc, int64_t batch, int slices,
                                int blocks_per_slice, hipStream_t s) {
  const int64_t Mp = MT * 32;
  const dim3 grid((unsigned)((N + 127) / 128), (unsigned)slices, (unsigned)batch);
  if (slices == 1) {
    hipLaunchKernelGGL((gemm_skinny_kernel<SK, ASYM, MT>), grid, dim3(256), 0, s, Ap, Bc, Bs, C, M, N, K, ldc, M * ldc,
                       (int64_t)0, blocks_per_slice);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((gemm_skinny_kernel<SK, ASYM, MT>), grid, dim3(256), 0, s, Ap, Bc, Bs, partial, M, N, K, N,
                     (int64_t)slices * Mp * N, Mp * N, blocks_per_slice);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)((M * N + 255) / 256), 1, (unsigned)batch), dim3(256), 0, s,
                     partial, C, M, N, Mp, ldc, slices);
  return hipGetLastError();
}

hipError_t launch_gemm_skinny_path(int scale_kind, bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                   const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                   int64_t ldc, int64_t batch, void* workspace, hipStream_t s,
                                   const KernelTimer& timer) {
  if (!skinny_path_supported(M, N, K)) return hipErrorInvalidValue;
  const int64_t Mp = 32 * skinny_row_tiles(M);
  uint16_t* Ap = reinterpret_cast<uint16_t*>(workspace);
  const size_t panel_bytes = ((size_t)(batch * Mp * K * 2) + 255) / 256 * 256;
  float* partial = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(workspace) + panel_bytes);
  int blocks_per_slice;
  const int slices = skinny_outer_slices((N + 127) / 128 * batch, K / kSkinnyBlockK, blocks_per_slice);
  hipError_t e = launch_expand_bf16(scale_kind, asym, 32, A_codes, A_scales, M, K, Mp, K, batch, false, Ap, s);
  if (e != hipSuccess) return e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  // E8M0 floor and round share the byte encoding
  const int sk = scale_kind == kScaleE8M0Round ? kScaleE8M0Floor : scale_kind;
  auto go = [&]<int SK, bool ASYM>() {
    switch ((int)(Mp / 32)) {
      case 1: return launch_skinny<SK, ASYM, 1>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
      case 2: return launch_skinny<SK, ASYM, 2>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
      case 3: return launch_skinny<SK, ASYM, 3>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
      case 4: return launch_skinny<SK, ASYM, 4>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
      case 6: return launch_skinny<SK, ASYM, 6>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
      default: return launch_skinny<SK, ASYM, 8>(Ap, B_codes, B_scales, C, partial, M, N, K, ldc, batch, slices, blocks_per_slice, s);
    }
  };
  if (sk == kScaleE5M2)
    e = asym ? go.template operator()<kScaleE5M2, true>() : go.template operator()<kScaleE5M2, false>();
  else if (sk == kScaleE4M3)
    e = asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>();
  else
    e = asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
  if (e != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

}  // namespace amx
