// Fully quantized GEMM for ASYMMETRIC power-of-two scales (Eq. 1 with E8M0 scales, Sec. 4.2 "PoT") on the block-scaled
// FP8 matrix instruction, one MFMA per block instead of the four of the sign-split FP4 kernel (gemm_fp4.hip).
//
// Merging. A group carries two power-of-two scales 2^sp, 2^sn (positive / negative elements). With the anchor
// a = max(sp, sn) every element is  elem * 2^(s_class - a)  times the block scale 2^a, and elem * 2^-d with
// elem in {.5,1,1.5,2,3,4,6} is an exact E5M2 number for d <= 13 (same two mantissa bits, exponent lowered by d).
// The merge kernel writes those E5M2 bytes and the anchor bytes; v_mfma_scale_f32_32x32x64_f8f6f4 with E5M2 operands
// then applies 2^(a_A + a_B) per 32-block, so every operand element is exact. Two things are not: (1) an ELEMENT whose
// merged value would fall below the E5M2 range (its class scale more than 2^13 below the anchor, counted per element:
// larger elements of such a class survive a binade or two longer than smaller ones) is flushed to zero: it is below
// 6 * 2^-14 of the group's scale unit while the other class reaches at least 4 units; (2) the instruction adds the 32
// products of a block in a fixed-point window below the largest of them, so a product far below the block's largest
// loses low bits: an absolute error of about 2^-22 of that largest product per block, whatever the sum is. Measured
// against the FP64 sums: 0 for classes 2^4 apart, 1.8e-5 for 2^8, 5.4e-5 for 2^12 (relative, in norm, random
// magnitudes). The sign-split and the FP6 kernels have neither effect.
//
// Layout. For 8-bit operands the instruction's 8-register operand of lane l = 32 * u + row holds, in registers
// 4 h .. 4 h + 3, the elements 16 u .. 16 u + 15 of the row's 32-block h of the K step of 64, and takes the block scale
// of 32-block h from lanes 32 h .. 32 h + 31 (probed on the machine; for FP4 operands a lane holds one whole block).
// The merge kernel writes "fragment-major" panels accordingly: per 32-row block and K block of 64, two KiB-sized
// halves [64 lanes][16 bytes], half h = 32-block h, lane 32 u + row = its elements 16 u .. 16 u + 15; the two halves
// are the two 128-bit LDS reads that fill an operand. Rows are padded to 256, K to 256 with zeros. Anchors:
// [row block][K / 256][64 lanes] words, byte q of the word of lane 32 h + row = the anchor of (row, 32-block h) in K
// stage 4 w + q. The GEMM kernel is gemm_bf16.hip's pipeline with one
// stage = K 64 = the same 32 KiB: ring of four LDS stages filled by direct-to-LDS loads, one barrier per stage.
#include "device_formats.h"
#include "gemm_common.h"
#include "kernels.h"

namespace amx {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMergeK = 256;  // K padding of the merged panels (4 stages of 64)

static int64_t merged_panel_bytes(int64_t rows_p, int64_t Kp) { return rows_p * Kp; }
static int64_t merged_scale_bytes(int64_t rows_p, int64_t Kp) { return (rows_p / 32) * (Kp / 256) * 256; }

size_t fp8m_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch) {
  const int64_t Kp = round_up(K, kMergeK), Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows);
  return (size_t)(batch * (merged_panel_bytes(Mp, Kp) + merged_panel_bytes(Np, Kp) + merged_scale_bytes(Mp, Kp) +
                           merged_scale_bytes(Np, Kp)));
}

// E5M2 byte of elem * 2^-d for the 3-bit magnitude code m (0 for m = 0 or when the exponent would leave the normal
// range), sign in bit 7. E5M2 patterns of .5,1,1.5,2,3,4,6: 0x38 0x3C 0x3E 0x40 0x42 0x44 0x46.
__device__ __forceinline__ uint32_t merged_byte(uint32_t nib, uint32_t d4_pos, uint32_t d4_neg) {
  const uint32_t m = nib & 7u, neg = nib >> 3;
  const uint32_t base = (uint32_t)(0x464442403E3C3800ull >> (8u * m)) & 255u;
  const uint32_t d4 = neg ? d4_neg : d4_pos;  // 4 * d: the exponent field starts at bit 2
  const uint32_t v = base >= d4 + 4u ? base - d4 : 0u;
  return (m ? v : 0u) | (neg << 7);
}

// grid: (Kp / 256, Rp / 32, batch); block 256 = 4 waves; wave w merges K stage 4 * blockIdx.x + w of one 32-row block:
// lane = 32 * h + row % 32 merges 32-block h of its row (and is the lane that supplies that block's anchor).
__global__ __launch_bounds__(256) void merge_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                    int64_t R, int64_t K, int64_t Rp, int64_t Kp,
                                                    uint8_t* __restrict__ panel, uint8_t* __restrict__ anchors) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t rb = blockIdx.y, b = blockIdx.z;
  const int64_t stage = (int64_t)blockIdx.x * 4 + wave;
  const int64_t r = rb * 32 + (lane & 31);
  const int64_t g = stage * 2 + (lane >> 5);
  const int64_t G = K >> 5;
  uint32_t w[4] = {0, 0, 0, 0};
  uint32_t sp = 0, sn = 0;
  if (r < R && g < G) {
    const uint4 c = *reinterpret_cast<const uint4*>(codes + (b * R + r) * (K >> 1) + g * 16);
    w[0] = c.x, w[1] = c.y, w[2] = c.z, w[3] = c.w;
    const uint32_t sb = *reinterpret_cast<const uint16_t*>(scales + ((b * R + r) * G + g) * 2);
    sp = sb & 255u, sn = sb >> 8;
  }
  const uint32_t anchor = sp > sn ? sp : sn;
  const uint32_t d4_pos = (anchor - sp) * 4u, d4_neg = (anchor - sn) * 4u;
  // half (lane / 32) of the fragment; elements 16 u .. 16 u + 15 go to lane slot 32 u + row
  uint8_t* half = panel + ((b * (Rp >> 5) + rb) * (Kp >> 6) + stage) * 2048 + (lane >> 5) * 1024 + (lane & 31) * 16;
#pragma unroll
  for (int u = 0; u < 2; ++u) {  // codes 16 u .. 16 u + 15 = words 2 u, 2 u + 1
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {  // output word q = 4 codes = half of input word 2 u + q / 2
      const uint32_t src = w[2 * u + (q >> 1)] >> (16 * (q & 1));
      o[q] = merged_byte(src & 15u, d4_pos, d4_neg) | (merged_byte((src >> 4) & 15u, d4_pos, d4_neg) << 8) |
             (merged_byte((src >> 8) & 15u, d4_pos, d4_neg) << 16) |
             (merged_byte((src >> 12) & 15u, d4_pos, d4_neg) << 24);
    }
    *reinterpret_cast<uint4*>(half + u * 512) = make_uint4(o[0], o[1], o[2], o[3]);
  }
  anchors[(((b * (Rp >> 5) + rb) * (Kp >> 8) + blockIdx.x) * 64 + lane) * 4 + wave] = (uint8_t)anchor;
}

// GLU: the gated-activation epilogue of store_glu_tiles() (gemm_common.h); C is then the BF16 output [M][ldc].
template <int WM, int WN, int FM, int FN, bool GLU = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_fp8m_kernel(const uint8_t* __restrict__ Ap,
                                                                 const uint8_t* __restrict__ Asc,
                                                                 const uint8_t* __restrict__ Bp,
                                                                 const uint8_t* __restrict__ Bsc, float* __restrict__ C,
                                                                 int64_t M, int64_t N, int64_t Mp, int64_t Np,
                                                                 int64_t Kp, int64_t ldc, int tiles_m, int tiles_n,
                                                                 int super_m) {
  using Cfg = TileCfg<WM, WN, FM, FN>;
  // separate arrays per stage: see gemm_bf16.hip
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

  const int nstages = (int)(Kp >> 6);  // multiple of 4
  const int nwords = nstages >> 2;
  const uint8_t* Abase = Ap + ((b * (Mp >> 5) + (int64_t)tm * (Cfg::kTileM / 32)) * nstages) * 2048;
  const uint8_t* Bbase = Bp + ((b * (Np >> 5) + (int64_t)tn * (Cfg::kTileN / 32)) * nstages) * 2048;
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Abase), 0, (Cfg::kTileM / 32) * nstages * 2048, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bbase), 0, (Cfg::kTileN / 32) * nstages * 2048, 0x00020000);
  // anchor words of this wave's row blocks: [row block][word][64 lanes] x 4 bytes
  const __amdgpu_buffer_rsrc_t Asr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Asc + ((b * (Mp >> 5) + (int64_t)tm * (Cfg::kTileM / 32) + wm * FM) * nwords) * 256), 0,
      FM * nwords * 256, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bsc + ((b * (Np >> 5) + (int64_t)tn * (Cfg::kTileN / 32) + wn * FN) * nwords) * 256), 0,
      FN * nwords * 256, 0x00020000);
  const int lane_off = lane * 16;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Load L of this wave for stage ST: KiB f = wave + kWaves * L of the stage; f < kFragsA: A row block f / 2, half
  // f % 2; otherwise the same for B.
  constexpr int kWaves = Cfg::kWaves, kFragsA = Cfg::kFragsA, kLoads = Cfg::kLoads;
#define AMX_ISSUE_LOAD(L, ST, DST)                                                                         \
  {                                                                                                        \
    const int f_ = wave + kWaves * (L);                                                                    \
    if ((L) < kFragsA / kWaves)                                                                            \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,     \
                                               ((f_ >> 1) * nstages + (ST)) * 2048 + (f_ & 1) * 1024, 0, 0); \
    else                                                                                                   \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                            \
          Br, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,                                          \
          (((f_ - kFragsA) >> 1) * nstages + (ST)) * 2048 + (f_ & 1) * 1024, 0, 0);                        \
  }
  // anchor words of 4 stages (word W) into register set SET
  uint32_t sa[2][FM], sb[2][FN];
#define AMX_LOAD_ANCHORS(SET, W)                                                                        \
  {                                                                                                     \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) sa[SET][i] =                                         \
        __builtin_amdgcn_raw_buffer_load_b32(Asr, lane * 4, (i * nwords + (W)) * 256, 0);               \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) sb[SET][j] =                                         \
        __builtin_amdgcn_raw_buffer_load_b32(Bsr, lane * 4, (j * nwords + (W)) * 256, 0);               \
  }

#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 0, lds0);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 1, lds1);
  AMX_LOAD_ANCHORS(0, 0);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 2, lds2);
  AMX_WAIT_VMCNT(kLoads);
  AMX_BARRIER();

  // A operand of step t in aR[t & 1] (read one step ahead), B operands of stage S in bR[S & 1] (read during S - 1)
  u32x4 aR[2][2], bR[2][FN][2];  // [..][half]
  const int offA = lane_off + (wm * FM) * 2 * kFragBytes;
  const int offB = lane_off + (kFragsA + (wn * FN) * 2) * kFragBytes;
#define AMX_RD(P) (*reinterpret_cast<const u32x4*>(P))
  aR[0][0] = AMX_RD(lds0 + offA);
  aR[0][1] = AMX_RD(lds0 + offA + kFragBytes);
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    bR[0][j][0] = AMX_RD(lds0 + offB + j * 2 * kFragBytes);
    bR[0][j][1] = AMX_RD(lds0 + offB + j * 2 * kFragBytes + kFragBytes);
  }
#define AMX_OPERAND(LO, HI) \
  i32x8 { (int)(LO).x, (int)(LO).y, (int)(LO).z, (int)(LO).w, (int)(HI).x, (int)(HI).y, (int)(HI).z, (int)(HI).w }

  // Stage S = stage Q (0..3, a literal: it selects the anchor byte) of the word in set SET; B operands in set BSET.
  // Step i: reads the A operand of step i + 1 (of the next stage's step 0 when i = FM - 1) and B operand i of the next
  // stage, issues its share of the direct-to-LDS loads of stage S + 3, then FN MFMAs. Stage 0 of a word first requests
  // the next word's anchors into the other set.
#define AMX_STAGE(S, SET, Q, BSET, CUR, NXT, FETCH)                                                              \
  {                                                                                                              \
    const int fetch_ = (S) + 3 < nstages ? (S) + 3 : nstages - 1;                                                \
    if constexpr ((Q) == 0) {                                                                                    \
      const int w_ = ((S) >> 2) + 1 < nwords ? ((S) >> 2) + 1 : nwords - 1;                                      \
      AMX_LOAD_ANCHORS((SET) ^ 1, w_);                                                                           \
    }                                                                                                            \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                             \
      {                                                                                                          \
        const uint8_t* src_ = i + 1 < FM ? (CUR) : (NXT);                                                        \
        const int i2 = (i + 1) % FM;                                                                             \
        aR[(i + 1) & 1][0] = AMX_RD(src_ + offA + i2 * 2 * kFragBytes);                                          \
        aR[(i + 1) & 1][1] = AMX_RD(src_ + offA + i2 * 2 * kFragBytes + kFragBytes);                             \
      }                                                                                                          \
      if (i < FN) {                                                                                              \
        bR[(BSET) ^ 1][i][0] = AMX_RD((NXT) + offB + i * 2 * kFragBytes);                                        \
        bR[(BSET) ^ 1][i][1] = AMX_RD((NXT) + offB + i * 2 * kFragBytes + kFragBytes);                           \
      }                                                                                                          \
      _Pragma("unroll") for (int l = i; l < kLoads; l += FM) AMX_ISSUE_LOAD(l, fetch_, FETCH);                   \
      {                                                                                                          \
        const i32x8 av = AMX_OPERAND(aR[i & 1][0], aR[i & 1][1]);                                                \
        _Pragma("unroll") for (int j = 0; j < FN; ++j) acc[i][j] =                                               \
            __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, AMX_OPERAND(bR[BSET][j][0], bR[BSET][j][1]),     \
                                                            acc[i][j], 1, 1, Q, (int)sa[SET][i], Q,              \
                                                            (int)sb[SET][j]);                                    \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    AMX_WAIT_VMCNT(kLoads);                                                                                      \
    AMX_BARRIER();                                                                                               \
  }
  static_assert(FM % 2 == 0 && FN <= FM, "operand rings assume an even number of steps and one B read per step");

  // (no branch inside the loop body: a conditional half makes the register allocator spill)
  int s = 0;
  for (; s + 8 <= nstages; s += 8) {
    AMX_STAGE(s, 0, 0, 0, lds0, lds1, lds3);
    AMX_STAGE(s + 1, 0, 1, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 2, 0, 2, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 3, 0, 3, 1, lds3, lds0, lds2);
    AMX_STAGE(s + 4, 1, 0, 0, lds0, lds1, lds3);
    AMX_STAGE(s + 5, 1, 1, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 6, 1, 2, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 7, 1, 3, 1, lds3, lds0, lds2);
  }
  if (s < nstages) {  // one more word of four stages
    AMX_STAGE(s, 0, 0, 0, lds0, lds1, lds3);
    AMX_STAGE(s + 1, 0, 1, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 2, 0, 2, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 3, 0, 3, 1, lds3, lds0, lds2);
  }
  AMX_WAIT_VMCNT(0);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_OPERAND
#undef AMX_RD
#undef AMX_LOAD_ANCHORS
#undef AMX_ISSUE_LOAD

  if constexpr (GLU) {
    // every wave is past its last fragment read: the operand stages become the waves' transposition space
    static_assert(Cfg::kWaves <= 4 && glu_stage_bytes<FM, FN>() <= Cfg::kStageBytes, "stage too small");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    AMX_BARRIER();
    const int w = wm * WN + wn;
    uint8_t* stage = w == 0 ? lds0 : w == 1 ? lds1 : w == 2 ? lds2 : lds3;
    store_glu_tiles<FM, FN>(acc, stage, reinterpret_cast<uint16_t*>(C) + b * M * ldc, M, N >> 1, ldc,
                            (int64_t)tm * Cfg::kTileM + wm * FM * 32, (int64_t)tn * Cfg::kTileN + wn * FN * 32);
  } else
    store_c_tiles<FM, FN>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * Cfg::kTileM + wm * FM * 32,
                          (int64_t)tn * Cfg::kTileN + wn * FN * 32);
}

hipError_t launch_gemm_fp8m_path(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                 const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc, int64_t batch,
                                 void* workspace, hipStream_t s, const KernelTimer& timer, bool glu) {
  const int64_t Kp = round_up(K, kMergeK), Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows);
  uint8_t* Ap = reinterpret_cast<uint8_t*>(workspace);
  uint8_t* Bp = Ap + batch * merged_panel_bytes(Mp, Kp);
  uint8_t* Asc = Bp + batch * merged_panel_bytes(Np, Kp);
  uint8_t* Bsc = Asc + batch * merged_scale_bytes(Mp, Kp);
  hipLaunchKernelGGL(merge_kernel, dim3((unsigned)(Kp / 256), (unsigned)(Mp / 32), (unsigned)batch), dim3(256), 0, s,
                     A_codes, A_scales, M, K, Mp, Kp, Ap, Asc);
  hipLaunchKernelGGL(merge_kernel, dim3((unsigned)(Kp / 256), (unsigned)(Np / 32), (unsigned)batch), dim3(256), 0, s,
                     B_codes, B_scales, N, K, Np, Kp, Bp, Bsc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  using Cfg = TileCfg<2, 2, 4, 4>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  if (glu)
    hipLaunchKernelGGL((gemm_fp8m_kernel<2, 2, 4, 4, true>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s,
                       Ap, Asc, Bp, Bsc, C, M, N, Mp, Np, Kp, ldc, tiles_m, tiles_n, super_m);
  else
    hipLaunchKernelGGL((gemm_fp8m_kernel<2, 2, 4, 4>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s, Ap,
                       Asc, Bp, Bsc, C, M, N, Mp, Np, Kp, ldc, tiles_m, tiles_n, super_m);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

}  // namespace amx
