// Fully quantized GEMM for power-of-two (E8M0) shared scales on the block-scaled FP4 matrix instruction
// v_mfma_scale_f32_32x32x64_f8f6f4: the packed E2M1 codes go to the matrix cores unchanged and the per-group scales
// ride along as the instruction's E8M0 block scales (one per 32 K-elements per row / column), so nothing is
// dequantized.
//
//   symmetric (MXFP4, Sec. 2.1 / Appendix B Algorithm 1): one MFMA per 32x32x64 block.
//   asymmetric (Eq. 1 with power-of-two scales, Sec. 4.2 "PoT"): a group is split by sign into two MXFP4 operands,
//     a = a_pos + a_neg with the other sign's codes zeroed, each carrying its own scale; the product of Sec. 4.3
//     becomes four MFMAs (pos*pos, pos*neg, neg*pos, neg*neg) whose block scales are the matching scale pairs.
//
// Operand fragment of the instruction for FP4: lane l holds row l%32, K block l/32 (32 codes = 16 bytes, element k in
// bits 4k+3:4k), and supplies the scale byte of that (row, K block) in a VGPR byte picked by the instruction's opsel.
// The canonical code layout already has those 16 bytes contiguous, so tiles are staged straight from the caller's
// arrays by direct-to-LDS buffer loads with per-lane offsets (no re-layout pass, no workspace).
// One stage = K slice of 128 (2 MFMA k-steps of 64): same byte count and LDS ring as the BF16 kernel.
#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ i32x8 as_operand(uint4 v) {
  i32x8 r = {(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};  // FP4 uses the first 4 of the 8 operand registers
  return r;
}

// Keep only the codes whose sign bit equals NEG (the others become +0): per nibble, 0xF where the sign bit is set.
template <bool NEG>
__device__ __forceinline__ uint32_t sign_class(uint32_t w) {
  const uint32_t neg = ((w >> 3) & 0x11111111u) * 15u;
  return NEG ? (w & neg) : (w & ~neg);
}
template <bool NEG>
__device__ __forceinline__ uint4 sign_class4(uint4 v) {
  return make_uint4(sign_class<NEG>(v.x), sign_class<NEG>(v.y), sign_class<NEG>(v.z), sign_class<NEG>(v.w));
}

template <int WM, int WN, int FM, int FN, bool ASYM>
__global__ __launch_bounds__(64 * WM * WN) void gemm_fp4_kernel(const uint8_t* __restrict__ Ac,
                                                                const uint8_t* __restrict__ As,
                                                                const uint8_t* __restrict__ Bc,
                                                                const uint8_t* __restrict__ Bs, float* __restrict__ C,
                                                                int64_t M, int64_t N, int64_t K, int64_t ldc,
                                                                int tiles_m, int tiles_n, int super_m) {
  using Cfg = TileCfg<WM, WN, FM, FN>;
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

  constexpr int kWaves = Cfg::kWaves, kFragsA = Cfg::kFragsA, kLoads = Cfg::kLoads, kTileM = Cfg::kTileM,
                kTileN = Cfg::kTileN;
  constexpr int kScaleBytes = ASYM ? 2 : 1;                    // per group
  const int row_bytes = (int)(K >> 1);                         // codes per row
  const int srow_bytes = (int)(K >> 5) * kScaleBytes;          // scale bytes per row
  const int rows_a = (int)(M - (int64_t)tm * kTileM < kTileM ? M - (int64_t)tm * kTileM : kTileM);
  const int rows_b = (int)(N - (int64_t)tn * kTileN < kTileN ? N - (int64_t)tn * kTileN : kTileN);

  // Raw buffer descriptors over this tile's rows: anything past the last valid row reads as zero. A zero scale byte
  // is 2^-127, so rows beyond M / N contribute products that vanish (and their outputs are never stored).
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Ac + (b * M + (int64_t)tm * kTileM) * row_bytes), 0, rows_a * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bc + (b * N + (int64_t)tn * kTileN) * row_bytes), 0, rows_b * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Asr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(As + (b * M + (int64_t)tm * kTileM) * srow_bytes), 0, rows_a * srow_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bs + (b * N + (int64_t)tn * kTileN) * srow_bytes), 0, rows_b * srow_bytes, 0x00020000);

  // Staging geometry. One direct-to-LDS load moves 16 rows x 64 bytes (4 lanes per row: the stage's 128 codes of that
  // row), so every lane quad reads one aligned 64-byte segment of its row. Its LDS image is [16 rows][4 chunks of
  // 16 bytes]; two loads make a row block of 32 rows x 64 bytes = 2 KiB. The chunk a lane fetches is permuted by the
  // row (chunk = slot ^ ((row >> 2) & 3)) so that the fragment reads below (32 consecutive rows, one chunk each) fall
  // on 16 distinct 16-byte bank groups per 16 lanes.
  const int kb = lane >> 5;  // K block (of 32 codes) of this lane inside a 64-wide k-step
  const int gather_off = (lane >> 2) * row_bytes + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);
  const int sgather_off = (lane & 31) * srow_bytes;
  // fragment read offsets inside a row block for k-step 0 and 1: row r = lane % 32 holds chunk c at slot c ^ ((r>>2)&3)
  const int rr = lane & 31;
  const int offk0 = rr * 64 + (((0 + kb) ^ ((rr >> 2) & 3)) << 4);
  const int offk1 = rr * 64 + (((2 + kb) ^ ((rr >> 2) & 3)) << 4);

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Load L of this wave for stage ST: half row block f = wave + kWaves * L (row block f / 2, rows 16 * (f % 2) ..);
  // f < kFragsA: operand A, otherwise B. Lands at DST + f KiB.
#define AMX_ISSUE_LOAD(L, ST, DST)                                                                              \
  {                                                                                                             \
    const int f_ = wave + kWaves * (L);                                                                         \
    if ((L) < kFragsA / kWaves)                                                                                 \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, gather_off,        \
                                               f_ * 16 * row_bytes + (ST) * 64, 0, 0);                          \
    else                                                                                                        \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, gather_off,        \
                                               (f_ - kFragsA) * 16 * row_bytes + (ST) * 64, 0, 0);              \
  }

  // Scale words, per lane and row block, for a PAIR of stages (8 groups of this lane's row): symmetric = 8 bytes
  // (one per group), asymmetric = 16 bytes ((pos, neg) per group). Two register sets alternate: pair P of stages
  // (2P, 2P+1) lives in set P & 1 and is requested two stages ahead.
  typedef uint32_t sword_t __attribute__((ext_vector_type(ASYM ? 4 : 2)));
  sword_t sa[2][FM], sb[2][FN];
#define AMX_LOAD_SCALES(SET, PAIR)                                                                                  \
  {                                                                                                                 \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                                \
      if constexpr (ASYM)                                                                                           \
        sa[SET][i] = __builtin_bit_cast(sword_t, __builtin_amdgcn_raw_buffer_load_b128(                             \
                                                     Asr, sgather_off + (PAIR) * 16, (wm * FM + i) * 32 * srow_bytes, 0)); \
      else                                                                                                          \
        sa[SET][i] = __builtin_bit_cast(sword_t, __builtin_amdgcn_raw_buffer_load_b64(                              \
                                                     Asr, sgather_off + (PAIR) * 8, (wm * FM + i) * 32 * srow_bytes, 0));  \
    }                                                                                                               \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) {                                                                \
      if constexpr (ASYM)                                                                                           \
        sb[SET][j] = __builtin_bit_cast(sword_t, __builtin_amdgcn_raw_buffer_load_b128(                             \
                                                     Bsr, sgather_off + (PAIR) * 16, (wn * FN + j) * 32 * srow_bytes, 0)); \
      else                                                                                                          \
        sb[SET][j] = __builtin_bit_cast(sword_t, __builtin_amdgcn_raw_buffer_load_b64(                              \
                                                     Bsr, sgather_off + (PAIR) * 8, (wn * FN + j) * 32 * srow_bytes, 0));  \
    }                                                                                                               \
  }
  constexpr int kScaleLoads = FM + FN;  // per pair of stages

  const int nstages = (int)(K >> 7);  // K is a multiple of 128 on this path
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 0, lds0);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, (nstages > 1 ? 1 : 0), lds1);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, (nstages > 2 ? 2 : nstages - 1), lds2);
  AMX_LOAD_SCALES(0, 0);
  AMX_WAIT_VMCNT(kLoads + kScaleLoads);  // everything older than the stage-2 loads and the scale loads has landed
  AMX_BARRIER();

  uint4 aR[4], bR[2][FN];
  const int baseA = (wm * FM) * 2 * kFragBytes;
  const int baseB = (kFragsA + (wn * FN) * 2) * kFragBytes;
  aR[0] = *reinterpret_cast<const uint4*>(lds0 + baseA + offk0);
  aR[1] = *reinterpret_cast<const uint4*>(lds0 + baseA + 2 * kFragBytes + offk0);
#pragma unroll
  for (int j = 0; j < FN; ++j) bR[0][j] = *reinterpret_cast<const uint4*>(lds0 + baseB + j * 2 * kFragBytes + offk0);

  // The MFMAs of step (KS, I) of stage Q (0 or 1) of a scale pair held in set SET. Scale byte selection:
  // symmetric: word Q = bytes (g0 g1 g2 g3) of the stage, shifted by 8*kb; k-step KS uses byte 2*KS (opsel);
  // asymmetric: word 2*Q + KS = bytes (p0 n0 p1 n1) of the k-step, shifted by 16*kb; pos = byte 0, neg = byte 1.
#define AMX_MMA(SET, Q, KS, I)                                                                                       \
  {                                                                                                                  \
    if constexpr (!ASYM) {                                                                                           \
      const int sav = (int)(sa[SET][I][Q] >> (8 * kb));                                                              \
      const i32x8 av = as_operand(aR[((KS) * FM + (I)) & 3]);                                                        \
      _Pragma("unroll") for (int j = 0; j < FN; ++j) {                                                               \
        const int sbv = (int)(sb[SET][j][Q] >> (8 * kb));                                                            \
        acc[I][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, as_operand(bR[(KS) & 1][j]), acc[I][j], 4,   \
                                                                    4, 2 * (KS), sav, 2 * (KS), sbv);                \
      }                                                                                                              \
    } else {                                                                                                         \
      const int sav = (int)(sa[SET][I][2 * (Q) + (KS)] >> (16 * kb));                                                \
      const uint4 araw = aR[((KS) * FM + (I)) & 3];                                                                  \
      const i32x8 ap = as_operand(sign_class4<false>(araw)), an = as_operand(sign_class4<true>(araw));              \
      _Pragma("unroll") for (int j = 0; j < FN; ++j) {                                                               \
        const int sbv = (int)(sb[SET][j][2 * (Q) + (KS)] >> (16 * kb));                                              \
        const i32x8 bp = as_operand(sign_class4<false>(bR[(KS) & 1][j])),                                            \
                    bn = as_operand(sign_class4<true>(bR[(KS) & 1][j]));                                             \
        acc[I][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ap, bp, acc[I][j], 4, 4, 0, sav, 0, sbv);        \
        acc[I][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ap, bn, acc[I][j], 4, 4, 0, sav, 1, sbv);        \
        acc[I][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(an, bp, acc[I][j], 4, 4, 1, sav, 0, sbv);        \
        acc[I][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(an, bn, acc[I][j], 4, 4, 1, sav, 1, sbv);        \
      }                                                                                                              \
    }                                                                                                                \
  }

  // Stage S = stage Q (0 / 1) of the scale pair in set SET; ring discipline as in gemm_bf16.hip. An even stage first
  // requests the scale words of the next pair (stages S + 2, S + 3) into the other set, whose previous contents
  // (stages S - 2, S - 1) are dead. Then each step reads fragments ahead, issues its share of the stage S + 3 loads and
  // multiplies.
#define AMX_STAGE(S, SET, Q, CUR, NXT, FETCH)                                                                     \
  {                                                                                                               \
    const int fetch_ = (S) + 3 < nstages ? (S) + 3 : nstages - 1;                                                 \
    if constexpr ((Q) == 0) AMX_LOAD_SCALES((SET) ^ 1, ((S) >> 1) + 1);                                           \
    _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                            \
      _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                            \
        const int t = ks * FM + i;                                                                                \
        {                                                                                                         \
          const int t2 = t + 2, ks2 = t2 / FM, i2 = t2 % FM;                                                      \
          const uint8_t* src_ = ks2 < 2 ? (CUR) : (NXT);                                                          \
          aR[t2 & 3] = *reinterpret_cast<const uint4*>(src_ + baseA + i2 * 2 * kFragBytes +                       \
                                                       ((ks2 & 1) ? offk1 : offk0));                              \
        }                                                                                                         \
        _Pragma("unroll") for (int jj = 2 * i; jj < 2 * i + 2; ++jj) {                                            \
          if (jj < FN) {                                                                                          \
            const uint8_t* src_ = ks == 0 ? (CUR) : (NXT);                                                        \
            bR[(ks + 1) & 1][jj] = *reinterpret_cast<const uint4*>(src_ + baseB + jj * 2 * kFragBytes +           \
                                                                   (((ks + 1) & 1) ? offk1 : offk0));             \
          }                                                                                                       \
        }                                                                                                         \
        _Pragma("unroll") for (int l = t; l < kLoads; l += 2 * FM) AMX_ISSUE_LOAD(l, fetch_, FETCH);              \
        if (ks == 0) AMX_MMA(SET, Q, 0, i) else AMX_MMA(SET, Q, 1, i);                                            \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
      }                                                                                                           \
    }                                                                                                             \
    /* younger than the stage S + 2 loads: this stage's scale loads (even stages) and its stage S + 3 loads */   \
    AMX_WAIT_VMCNT(kLoads + ((Q) == 0 ? kScaleLoads : 0));                                                        \
    AMX_BARRIER();                                                                                                \
  }

  int s = 0;
  for (; s + 4 <= nstages; s += 4) {
    AMX_STAGE(s, 0, 0, lds0, lds1, lds3);
    AMX_STAGE(s + 1, 0, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 2, 1, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 3, 1, 1, lds3, lds0, lds2);
  }
  // up to 3 remaining stages (K / 128 need not be a multiple of 4)
  if (s < nstages) AMX_STAGE(s, 0, 0, lds0, lds1, lds3);
  if (s + 1 < nstages) AMX_STAGE(s + 1, 0, 1, lds1, lds2, lds0);
  if (s + 2 < nstages) AMX_STAGE(s + 2, 1, 0, lds2, lds3, lds1);
  AMX_WAIT_VMCNT(0);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_MMA
#undef AMX_LOAD_SCALES
#undef AMX_ISSUE_LOAD

  float* Cb = C + b * M * ldc;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int64_t col = (int64_t)tn * kTileN + (wn * FN + j) * 32 + (lane & 31);
      const int64_t row0 = (int64_t)tm * kTileM + (wm * FM + i) * 32 + 4 * (lane >> 5);
      if (col < N) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t row = row0 + 8 * (v >> 2) + (v & 3);
          if (row < M) __builtin_nontemporal_store(acc[i][j][v], Cb + row * ldc + col);
        }
      }
    }
  }
}

bool fp4_path_supported(int64_t M, int64_t N, int64_t K) {
  // K in whole stages; per-tile byte offsets (256 rows x K/2 bytes, 256 rows x K/16 bytes) must fit the 32-bit
  // buffer offsets
  return K % 128 == 0 && K <= (1 << 22) && M > 0 && N > 0;
}

template <bool ASYM>
static hipError_t launch_fp4(int64_t M, int64_t N, int64_t K, const uint8_t* Ac, const uint8_t* As, const uint8_t* Bc,
                             const uint8_t* Bs, float* C, int64_t ldc, int64_t batch, hipStream_t s,
                             const KernelTimer& timer) {
  using Cfg = TileCfg<2, 2, 4, 4>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  hipError_t e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_fp4_kernel<2, 2, 4, 4, ASYM>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s, Ac,
                     As, Bc, Bs, C, M, N, K, ldc, tiles_m, tiles_n, super_m);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

hipError_t launch_gemm_fp4_path(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                int64_t ldc, int64_t batch, hipStream_t s, const KernelTimer& timer) {
  return asym ? launch_fp4<true>(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, s, timer)
              : launch_fp4<false>(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, s, timer);
}

}  // namespace amx
