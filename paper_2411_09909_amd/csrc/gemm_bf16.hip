// Fully quantized GEMM for scale formats whose values are not powers of two (FP8 E5M2, Sec. 4.2) and for the
// sign-asymmetric formats (Eq. 1, Sec. 4.3).
//
// A dequantized element is elem * S_class with elem in {0,.5,1,1.5,2,3,4,6} and S = (1 + m/4) * 2^e: up to 5
// significant bits (3 * 7 = 21; 6 bits with the 3 mantissa bits of an E4M3 scale, 3 * 15 = 45), which FP8/FP6/FP4
// MFMA operands cannot hold but BF16 holds exactly. Groups of 16, 64 or 128 elements, which do not match the 32-long
// blocks of the block-scaled instructions, also come here whatever their scale format. The GEMM is
// therefore run on the BF16 MFMA (v_mfma_f32_32x32x16_bf16) with exact operands and FP32 accumulation:
//
//   1. expand kernel: codes + scale pair -> BF16, written into "fragment-major" panels in the workspace:
//        panel[row_block of 32][k_block of 16][lane 0..63][8 BF16],  lane = 32 * (k / 8 % 2) + row % 32,
//      which is exactly the register image of one MFMA operand (lane l holds row l%32, k = 8*(l/32) .. +7).
//      Rows are padded to a multiple of 256 and K to a multiple of 128 with zeros.
//   2. GEMM kernel: every operand fragment is one contiguous KiB in the workspace, so staging global -> LDS is a
//      linear copy and LDS -> register reads are conflict-free 128-bit reads at lane * 16.

#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

size_t bf16_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch) {
  const int64_t Kp = round_up(K, kPanelK);
  return (size_t)(batch * (round_up(M, kPanelRows) + round_up(N, kPanelRows)) * Kp * 2);
}

size_t bf16_panel_bytes(int64_t rows, int64_t K) { return (size_t)(round_up(rows, kPanelRows) * round_up(K, kPanelK) * 2); }

// ------------------------------------------------------------------------------------------------ expand ----------
// grid: (ceil(Kp / 256), Rp / 32, batch); block 256 = 4 waves. A workgroup expands one 32-row block over a K span of
// 256, i.e. whole 128-byte lines of every code row (neighbouring workgroups run on different XCDs with separate L2s,
// so a line split between two of them would be fetched from HBM twice); wave w takes the 64-wide slice w of the span:
// lane = 32 * group_in_slice + row_in_block. The 16 fragments a workgroup writes are contiguous in the panel.
// F16: the panel holds FP16 values biased by 2^-3 instead of BF16 (FP8-E5M2 scales only: every such value lies in
// [2^-20, 43008] and has at most 5 significant bits, so it is an FP16 number, subnormals included).
// PERMUTE: within every block of 32 along K, the fragment of k-step j (0, 1) holds, in lane half h, the elements
// 16 j + 4 h + {0, 1, 2, 3, 8, 9, 10, 11} instead of 16 j + 8 h + {0 .. 7}. That is the order in which the rows of a
// 32x32 MFMA accumulator sit in a lane's registers, so an accumulator tile can be fed back as the other operand of a
// product over those rows without a transpose (the fused attention kernel multiplies probabilities with V this way).
// HALF_LINE: within every block of 256 along K (8 groups), k-step s (0 .. 15) holds, in lane half h, the 8 elements
// s % 4 of group 4 h + s / 4 instead of the 8 elements h of the 16 that follow 16 s: a lane half then draws all its
// 16 k-steps from one contiguous half (64 bytes of codes) of the block. The few-rows kernel reads its B operand in
// that order straight from the packed codes and needs A to match (a product sums over k in any order).
template <int SCALE_KIND, bool ASYM, bool F16, bool PERMUTE = false, bool HALF_LINE = false>
__global__ __launch_bounds__(256) void expand_kernel(const uint8_t* __restrict__ codes,
                                                     const uint8_t* __restrict__ scales, int64_t R, int64_t K,
                                                     int64_t Rp, int64_t Kp, int gs_log2,
                                                     uint16_t* __restrict__ panel) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t rb = blockIdx.y;
  const int64_t slice = (int64_t)blockIdx.x * 4 + wave;  // 64-wide K slice
  if (slice * 64 >= Kp) return;
  const int64_t r = rb * 32 + (lane & 31);
  const int64_t g = slice * 2 + (lane >> 5);  // the lane's block of 32 elements
  const int64_t b = blockIdx.z;
  uint32_t w[4] = {0, 0, 0, 0};
  // scales of the first and of the second 16 elements of the block (they differ only for groups of 16)
  float s_pos[2] = {0.f, 0.f}, s_neg[2] = {0.f, 0.f};
  if (r < R && g < (K >> 5)) {
    const uint4 c = *reinterpret_cast<const uint4*>(codes + (b * R + r) * (K >> 1) + g * 16);
    w[0] = c.x, w[1] = c.y, w[2] = c.z, w[3] = c.w;
    const int64_t row_groups = (b * R + r) * groups_per_row(K, gs_log2);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h == 1 && gs_log2 != 4) {
        s_pos[1] = s_pos[0], s_neg[1] = s_neg[0];
        break;
      }
      const int64_t gi = row_groups + ((g * 32 + h * 16) >> gs_log2);
      if constexpr (ASYM) {
        const uint32_t sb = *reinterpret_cast<const uint16_t*>(scales + gi * 2);
        s_pos[h] = scale_value<SCALE_KIND>(sb & 255u);
        s_neg[h] = scale_value<SCALE_KIND>(sb >> 8);
      } else {
        s_pos[h] = s_neg[h] = scale_value<SCALE_KIND>(scales[gi]);
      }
    }
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    s_pos[h] *= F16 ? 0.0625f : 0.5f;
    s_neg[h] *= F16 ? -0.0625f : -0.5f;
  }
  uint16_t* dst = panel + ((b * (Rp >> 5) + rb) * (Kp >> 4) + slice * 4 + (lane >> 5) * 2) * 512;
  uint32_t o[4][4];  // run t of 8 elements of the block -> 4 registers of 2 values
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t n0 = (w[t] >> (8 * j)) & 15u, n1 = (w[t] >> (8 * j + 4)) & 15u;
      const float v0 = (float)e2m1_twice(n0 & 7u) * ((n0 & 8u) ? s_neg[t >> 1] : s_pos[t >> 1]);
      const float v1 = (float)e2m1_twice(n1 & 7u) * ((n1 & 8u) ? s_neg[t >> 1] : s_pos[t >> 1]);
      if constexpr (F16)
        o[t][j] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(v0, v1));  // exact, see above
      else
        o[t][j] = (f2u(v0) >> 16) | (f2u(v1) & 0xFFFF0000u);  // truncation is exact: <= 6 significant bits
    }
  }
  if constexpr (HALF_LINE) {
    const int64_t blk = g >> 3;
    const int gl = (int)(g & 7);
    uint16_t* d2 = panel + ((b * (Rp >> 5) + rb) * (Kp >> 4) + blk * 16 + (gl & 3) * 4) * 512 +
                   ((gl >> 2) * 32 + (lane & 31)) * 8;
#pragma unroll
    for (int t = 0; t < 4; ++t) *reinterpret_cast<uint4*>(d2 + t * 512) = make_uint4(o[t][0], o[t][1], o[t][2], o[t][3]);
    return;
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {  // k block (t / 2), lane half (t % 2) of the block's two fragments
    uint4 out;
    if constexpr (PERMUTE)
      out = make_uint4(o[t & 2][2 * (t & 1)], o[t & 2][2 * (t & 1) + 1], o[(t & 2) + 1][2 * (t & 1)],
                       o[(t & 2) + 1][2 * (t & 1) + 1]);
    else
      out = make_uint4(o[t][0], o[t][1], o[t][2], o[t][3]);
    *reinterpret_cast<uint4*>(dst + (t >> 1) * 512 + ((t & 1) * 32 + (lane & 31)) * 8) = out;
  }
}

// ------------------------------------------------------------------------------------------------ GEMM ------------
// Tile configuration, stage ring and supertile order: gemm_common.h. Here one stage is a K slice of 32.

// SCALED: the result is multiplied by the product of the operands' tensor-wise scales alpha_a[0] * alpha_b[0]
// (Sec. 5.3, double scaling), read from device memory after the main loop.
// GLU: the gated-activation epilogue of store_glu_tiles() instead of the FP32 store: C is then the BF16 output
// [M][ldc] with N / 2 columns.
template <int WM, int WN, int FM, int FN, bool SCALED, bool GLU = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(const uint16_t* __restrict__ Ap,
                                                                 const uint16_t* __restrict__ Bp, float* __restrict__ C,
                                                                 int64_t M, int64_t N, int64_t Mp, int64_t Np,
                                                                 int64_t Kp, int64_t ldc, int tiles_m, int tiles_n,
                                                                 int super_m, const float* __restrict__ alpha_a,
                                                                 const float* __restrict__ alpha_b) {
  using Cfg = TileCfg<WM, WN, FM, FN>;
  // Four separate arrays rather than one ring buffer: the compiler then knows that a direct-to-LDS load into one
  // stage cannot alias the fragment reads of another and does not serialise them.
  __shared__ __attribute__((aligned(1024))) uint8_t lds0[Cfg::kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds1[Cfg::kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds2[Cfg::kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds3[Cfg::kStageBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int64_t b = blockIdx.z;

  int tm, tn;
  if (!tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, super_m, tm, tn)) return;  // uniform, before any barrier

  // Buffer descriptors over this tile's slice of each panel: (tile rows / 32) row blocks x kblocks fragments of 1 KiB.
  // Raw buffer (stride 0), so reads past num_records return zero instead of faulting.
  const int kblocks = (int)(Kp >> 4);
  const uint8_t* Abase = reinterpret_cast<const uint8_t*>(Ap) +
                         ((b * (Mp >> 5) + (int64_t)tm * (Cfg::kTileM / 32)) * kblocks) * kFragBytes;
  const uint8_t* Bbase = reinterpret_cast<const uint8_t*>(Bp) +
                         ((b * (Np >> 5) + (int64_t)tn * (Cfg::kTileN / 32)) * kblocks) * kFragBytes;
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Abase), 0, (Cfg::kTileM / 32) * kblocks * kFragBytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bbase), 0, (Cfg::kTileN / 32) * kblocks * kFragBytes, 0x00020000);
  const int lane_off = lane * 16;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Load number L (0 .. kLoads-1) of this wave for K stage ST into ring slot array DST: fragment f = wave + kWaves * L
  // of the stage; f < kFragsA: A row block f / 2, k block f % 2; otherwise the same for B. One contiguous KiB of the
  // panel goes to DST + f KiB (the hardware adds lane * 16 on the LDS side).
  // (local copies of the tile constants: naming Cfg:: members directly inside the builtin's arguments trips the host
  // pass of the compiler, which then drops the kernel's launch stub)
  constexpr int kWaves = Cfg::kWaves, kFragsA = Cfg::kFragsA, kLoads = Cfg::kLoads;
#define AMX_ISSUE_LOAD(L, ST, DST)                                                                         \
  {                                                                                                        \
    const int f_ = wave + kWaves * (L);                                                                    \
    if ((L) < kFragsA / kWaves) /* decided at compile time once the loops are unrolled */                  \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,     \
                                               ((f_ >> 1) * kblocks + (ST) * 2 + (f_ & 1)) * kFragBytes,   \
                                               0, 0);                                                      \
    else                                                                                                   \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                            \
          Br, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,                                          \
          (((f_ - kFragsA) >> 1) * kblocks + (ST) * 2 + (f_ & 1)) * kFragBytes, 0, 0);                     \
  }

  const int nstages = (int)(Kp / 32);  // one stage = a K slice of 32 BF16 (2 MFMA k-steps); multiple of 4
  // prologue: 3 stages in flight; stages 0 and 1 must have landed before the first fragment reads
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 0, lds0);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 1, lds1);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 2, lds2);
  AMX_WAIT_VMCNT(kLoads);
  AMX_BARRIER();

  // register rings: the A fragment for step t lives in aR[t & 3] (read two steps ahead), the B fragments of k-step ks
  // in bR[ks & 1] (read during the previous k-step)
  bf16x8 aR[4], bR[2][FN];
  const int offA = lane_off + (wm * FM) * 2 * kFragBytes;
  const int offB = lane_off + (Cfg::kFragsA + (wn * FN) * 2) * kFragBytes;
  aR[0] = *reinterpret_cast<const bf16x8*>(lds0 + offA);
  aR[1] = *reinterpret_cast<const bf16x8*>(lds0 + offA + 2 * kFragBytes);
#pragma unroll
  for (int j = 0; j < FN; ++j) bR[0][j] = *reinterpret_cast<const bf16x8*>(lds0 + offB + j * 2 * kFragBytes);

  // One stage: 2 k-steps x FM steps; a step issues the fragment reads needed two steps (A) or one k-step (B) later,
  // its share of the direct-to-LDS loads for stage S + 3, then FN MFMAs. CUR / NXT are the ring arrays of stage S and
  // S + 1, FETCH the one stage S + 3 lands in (last read during stage S - 1). Past the end of K the fetch is pointed
  // at the last real stage instead of being skipped: it lands in a slot nobody reads any more and the body stays free
  // of branches.
#define AMX_STAGE(S, CUR, NXT, FETCH)                                                                                \
  {                                                                                                                  \
    const int fetch_ = (S) + 3 < nstages ? (S) + 3 : nstages - 1;                                                    \
    _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                               \
      _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                               \
        const int t = ks * FM + i;                                                                                   \
        {                                                                                                            \
          const int t2 = t + 2, ks2 = t2 / FM, i2 = t2 % FM;                                                         \
          const uint8_t* src_ = ks2 < 2 ? (CUR) : (NXT);                                                             \
          aR[t2 & 3] = *reinterpret_cast<const bf16x8*>(src_ + offA + (i2 * 2 + (ks2 & 1)) * kFragBytes);           \
        }                                                                                                            \
        _Pragma("unroll") for (int jj = 2 * i; jj < 2 * i + 2; ++jj) {                                               \
          if (jj < FN) {                                                                                             \
            const uint8_t* src_ = ks == 0 ? (CUR) : (NXT);                                                           \
            bR[(ks + 1) & 1][jj] =                                                                                   \
                *reinterpret_cast<const bf16x8*>(src_ + offB + (jj * 2 + ((ks + 1) & 1)) * kFragBytes);             \
          }                                                                                                          \
        }                                                                                                            \
        _Pragma("unroll") for (int l = t; l < kLoads; l += 2 * FM) AMX_ISSUE_LOAD(l, fetch_, FETCH);            \
        _Pragma("unroll") for (int j = 0; j < FN; ++j) acc[i][j] =                                                   \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(aR[t & 3], bR[ks & 1][j], acc[i][j], 0, 0, 0);                   \
        __builtin_amdgcn_sched_barrier(0);                                                                           \
      }                                                                                                              \
    }                                                                                                                \
    /* stage S + 2 must be complete in LDS for every wave before stage S + 1 starts reading ahead into it; the same  \
       barrier tells every wave that stage S is no longer read, so its slot may be refilled during stage S + 1 */    \
    AMX_WAIT_VMCNT(kLoads);                                                                                     \
    AMX_BARRIER();                                                                                                   \
  }

  for (int s = 0; s < nstages; s += 4) {
    AMX_STAGE(s, lds0, lds1, lds3);
    AMX_STAGE(s + 1, lds1, lds2, lds0);
    AMX_STAGE(s + 2, lds2, lds3, lds1);
    AMX_STAGE(s + 3, lds3, lds0, lds2);
  }
  AMX_WAIT_VMCNT(0);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_ISSUE_LOAD

  if constexpr (GLU) {
    // every wave is past its last fragment read: the operand stages become the waves' transposition space
    static_assert(glu_stage_bytes<FM, FN>() * ((Cfg::kWaves + 3) / 4) <= Cfg::kStageBytes, "stage too small");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    AMX_BARRIER();
    const int w = wm * WN + wn;
    uint8_t* stage = ((w & 3) == 0 ? lds0 : (w & 3) == 1 ? lds1 : (w & 3) == 2 ? lds2 : lds3) +
                     (w >> 2) * glu_stage_bytes<FM, FN>();
    store_glu_tiles<FM, FN>(acc, stage, reinterpret_cast<uint16_t*>(C) + b * M * ldc, M, N >> 1, ldc,
                            (int64_t)tm * Cfg::kTileM + wm * FM * 32, (int64_t)tn * Cfg::kTileN + wn * FN * 32);
  } else if constexpr (SCALED)
    store_c_tiles<FM, FN, 0, true>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * Cfg::kTileM + wm * FM * 32,
                                   (int64_t)tn * Cfg::kTileN + wn * FN * 32, alpha_a[0] * alpha_b[0]);
  else
    store_c_tiles<FM, FN>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * Cfg::kTileM + wm * FM * 32,
                          (int64_t)tn * Cfg::kTileN + wn * FN * 32);
}

template <int SK, bool ASYM, bool F16 = false>
static hipError_t launch_expand(const uint8_t* codes, const uint8_t* scales, int64_t R, int64_t K, int64_t Rp,
                                int64_t Kp, int gs_log2, int64_t batch, uint16_t* panel, hipStream_t s) {
  hipLaunchKernelGGL((expand_kernel<SK, ASYM, F16>), dim3((unsigned)((Kp + 255) / 256), (unsigned)(Rp / 32), (unsigned)batch),
                     dim3(256), 0, s, codes, scales, R, K, Rp, Kp, gs_log2, panel);
  return hipGetLastError();
}

static hipError_t expand_dispatch(int scale_kind, bool asym, int gs_log2, const uint8_t* codes, const uint8_t* scales,
                                  int64_t R, int64_t K, int64_t Rp, int64_t Kp, int64_t batch, uint16_t* panel,
                                  hipStream_t s) {
  if (scale_kind == kScaleE5M2)
    return asym ? launch_expand<kScaleE5M2, true>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s)
                : launch_expand<kScaleE5M2, false>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s);
  if (scale_kind == kScaleE4M3)
    return asym ? launch_expand<kScaleE4M3, true>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s)
                : launch_expand<kScaleE4M3, false>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s);
  return asym ? launch_expand<kScaleE8M0Floor, true>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s)
              : launch_expand<kScaleE8M0Floor, false>(codes, scales, R, K, Rp, Kp, gs_log2, batch, panel, s);
}

hipError_t launch_expand_bf16(int scale_kind, bool asym, int64_t group_size, const uint8_t* codes,
                              const uint8_t* scales, int64_t R, int64_t K, int64_t Rp, int64_t Kp, int64_t batch,
                              bool permute, uint16_t* panel, hipStream_t s) {
  const int gs_log2 = group_log2(group_size);
  if (gs_log2 < 0 || !group_divides(K, group_size) || K % 32 != 0 || Rp % 32 != 0 || Kp % 64 != 0) return hipErrorInvalidValue;
  if (!permute) return expand_dispatch(scale_kind, asym, gs_log2, codes, scales, R, K, Rp, Kp, batch, panel, s);
  const dim3 grid((unsigned)((Kp + 255) / 256), (unsigned)(Rp / 32), (unsigned)batch);
  auto go = [&]<int SK, bool ASYM>() {
    hipLaunchKernelGGL((expand_kernel<SK, ASYM, false, true>), grid, dim3(256), 0, s, codes, scales, R, K, Rp, Kp,
                       gs_log2, panel);
    return hipGetLastError();
  };
  if (scale_kind == kScaleE5M2) {
    // FP16 with a bias of 2^-3 (every element * scale / 8 is an FP16 number): the probabilities it is multiplied with
    // come out of the attention kernel's cast as FP16 for this scale format
    auto go16 = [&]<bool ASYM>() {
      hipLaunchKernelGGL((expand_kernel<kScaleE5M2, ASYM, true, true>), grid, dim3(256), 0, s, codes, scales, R, K, Rp,
                         Kp, gs_log2, panel);
      return hipGetLastError();
    };
    return asym ? go16.template operator()<true>() : go16.template operator()<false>();
  }
  if (scale_kind == kScaleE4M3) return asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>();
  return asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
}

hipError_t launch_expand_half_line(int scale_kind, bool asym, const uint8_t* codes, const uint8_t* scales, int64_t R,
                                   int64_t K, int64_t Rp, int64_t batch, uint16_t* panel, hipStream_t s) {
  if (K % 256 != 0 || Rp % 32 != 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(K / 256), (unsigned)(Rp / 32), (unsigned)batch);
  auto go = [&]<int SK, bool ASYM, bool F16>() {
    hipLaunchKernelGGL((expand_kernel<SK, ASYM, F16, false, true>), grid, dim3(256), 0, s, codes, scales, R, K, Rp, K,
                       5, panel);
    return hipGetLastError();
  };
  if (scale_kind == kScaleE5M2)
    return asym ? go.template operator()<kScaleE5M2, true, true>() : go.template operator()<kScaleE5M2, false, true>();
  if (scale_kind == kScaleE4M3)
    return asym ? go.template operator()<kScaleE4M3, true, false>() : go.template operator()<kScaleE4M3, false, false>();
  return asym ? go.template operator()<kScaleE8M0Floor, true, false>()
              : go.template operator()<kScaleE8M0Floor, false, false>();
}

hipError_t launch_expand_f16_e5m2(bool asym, const uint8_t* codes, const uint8_t* scales, int64_t R, int64_t K,
                                  int64_t Rp, int64_t Kp, int64_t batch, uint16_t* panel, hipStream_t s) {
  return asym ? launch_expand<kScaleE5M2, true, true>(codes, scales, R, K, Rp, Kp, 5, batch, panel, s)
              : launch_expand<kScaleE5M2, false, true>(codes, scales, R, K, Rp, Kp, 5, batch, panel, s);
}

template <int WM, int WN, int FM, int FN>
static hipError_t launch_tiles(const uint16_t* Ap, const uint16_t* Bp, float* C, int64_t M, int64_t N, int64_t Mp,
                               int64_t Np, int64_t Kp, int64_t ldc, int64_t batch, const float* alpha_a,
                               const float* alpha_b, bool glu, hipStream_t s) {
  using Cfg = TileCfg<WM, WN, FM, FN>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  if (glu)
    hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, FM, FN, false, true>), dim3(grid, 1, (unsigned)batch),
                       dim3(Cfg::kThreads), 0, s, Ap, Bp, C, M, N, Mp, Np, Kp, ldc, tiles_m, tiles_n, super_m, alpha_a,
                       alpha_b);
  else if (alpha_a && alpha_b)
    hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, FM, FN, true>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0,
                       s, Ap, Bp, C, M, N, Mp, Np, Kp, ldc, tiles_m, tiles_n, super_m, alpha_a, alpha_b);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, FM, FN, false>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads),
                       0, s, Ap, Bp, C, M, N, Mp, Np, Kp, ldc, tiles_m, tiles_n, super_m, alpha_a, alpha_b);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16_path(int scale_kind, bool asym, int64_t group_size, int64_t M, int64_t N, int64_t K,
                                 const uint8_t* A_codes, const uint8_t* A_scales, const uint8_t* B_codes,
                                 const uint8_t* B_scales, const float* A_tensor_pair, const float* B_tensor_pair,
                                 float* C, int64_t ldc, int64_t batch, void* workspace, int tile, hipStream_t s,
                                 const KernelTimer& timer, bool glu, const void* B_panel) {
  const int gs_log2 = group_log2(group_size);
  if (gs_log2 < 0 || !group_divides(K, group_size) || K % 32 != 0) return hipErrorInvalidValue;
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows), Kp = round_up(K, kPanelK);
  uint16_t* Ap = reinterpret_cast<uint16_t*>(workspace);
  const uint16_t* Bp = B_panel ? reinterpret_cast<const uint16_t*>(B_panel) : Ap + batch * Mp * Kp;
  hipError_t e = expand_dispatch(scale_kind, asym, gs_log2, A_codes, A_scales, M, K, Mp, Kp, batch, Ap, s);
  if (e != hipSuccess) return e;
  if (!B_panel) {  // (a panel the caller expanded once: launch_expand_b_panel)
    e = expand_dispatch(scale_kind, asym, gs_log2, B_codes, B_scales, N, K, Np, Kp, batch, Ap + batch * Mp * Kp, s);
    if (e != hipSuccess) return e;
  }
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  // Tile shape. 256 x 256 (4 waves of 128 x 128) has the least operand traffic and LDS reads per MFMA and is what
  // large problems use; a problem with fewer such tiles than the chip has CUs, or with one side much smaller than a
  // tile, finishes sooner with 256 x 128 or 64 x 256 tiles that fill the CUs. The choice minimises
  // (rounds of 256 workgroups) x (measured cost of one tile relative to a 256 x 256 one: 0.6 and 0.4), and leaves
  // 256 x 256 only for a predicted gain of more than 15 %. A caller's option (tile != 0) overrides it.
  auto rounds = [&](int64_t tile_m, int64_t tile_n) {
    const int64_t tiles = ((M + tile_m - 1) / tile_m) * ((N + tile_n - 1) / tile_n) * batch;
    return (double)((tiles + 255) / 256);
  };
  if (tile == 0) {
    const double est1 = rounds(256, 256), est2 = 0.6 * rounds(256, 128), est3 = 0.4 * rounds(64, 256);
    const bool ok3 = est3 < 0.85 * est1;
    const bool ok2 = est2 < 0.85 * est1 && M > 256;  // (with a single row of 256-row tiles the 64-row tile was never worse)
    tile = ok3 && (!ok2 || est3 <= est2) ? 3 : ok2 ? 2 : 1;
  }
  if (tile == 2)
    e = launch_tiles<4, 1, 2, 4>(Ap, Bp, C, M, N, Mp, Np, Kp, ldc, batch, A_tensor_pair, B_tensor_pair, glu, s);  // 256 x 128
  else if (tile == 3)
    e = launch_tiles<1, 4, 2, 2>(Ap, Bp, C, M, N, Mp, Np, Kp, ldc, batch, A_tensor_pair, B_tensor_pair, glu, s);  // 64 x 256
  else
    e = launch_tiles<2, 2, 4, 4>(Ap, Bp, C, M, N, Mp, Np, Kp, ldc, batch, A_tensor_pair, B_tensor_pair, glu, s);
  if (e != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

hipError_t launch_expand_b_panel(int scale_kind, bool asym, int64_t group_size, int64_t N, int64_t K,
                                 const uint8_t* B_codes, const uint8_t* B_scales, void* panel, hipStream_t s) {
  const int gs_log2 = group_log2(group_size);
  if (gs_log2 < 0 || !group_divides(K, group_size) || K % 32 != 0) return hipErrorInvalidValue;
  return expand_dispatch(scale_kind, asym, gs_log2, B_codes, B_scales, N, K, round_up(N, kPanelRows), round_up(K, kPanelK),
                         1, reinterpret_cast<uint16_t*>(panel), s);
}

}  // namespace amx
