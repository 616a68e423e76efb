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
// The canonical code layout already has those 16 bytes contiguous, so the code tiles are staged straight from the
// caller's arrays by direct-to-LDS buffer loads with per-lane offsets (no re-layout of the codes).
// The scale bytes are different: a lane needs the 8 bytes of ITS row for the stage, and in the canonical layout the 32
// rows of a fragment lie a whole scale row apart, so a wave's fetch would touch 32 cache lines for 256 useful bytes,
// 256 line requests per wave and stage against the 128 of the codes themselves. That gather kept the vector memory
// path busy and the matrix pipe waiting (measured: the kernel with nothing but its MFMAs and these loads took 0.40 ms
// at the headline shape, 0.31 ms with the loads taken out). A small pass (scale_pack_kernel) therefore re-lays the
// scale bytes into the workspace in the order the waves read them, and a wave fetches the scales of its four row
// blocks for a stage with two (asymmetric: four) fully coalesced 16-byte loads.
#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef int i32x8 __attribute__((ext_vector_type(8)));
// 16 bytes of codes as one native vector: a fragment read is then a single load in the compiler's eyes and keeps the
// information which LDS array it reads (a struct of four words is read as four loads, three of which lose it, and the
// compiler then waits for every direct-to-LDS load in flight before each read)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ i32x8 as_operand(u32x4 v) {
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
__device__ __forceinline__ u32x4 sign_class4(u32x4 v) {
  u32x4 r = {sign_class<NEG>(v.x), sign_class<NEG>(v.y), sign_class<NEG>(v.z), sign_class<NEG>(v.w)};
  return r;
}

// Packed scales: [batch][rows / 128][stage = K / 256][row r of 32][row block i of 4][8 groups][1 or 2 bytes]. Entry
// (r, i) of row group q is row 128 q + 32 i + r; rows beyond the operand and groups beyond K hold byte 0 (2^-127: the
// products of the zero codes staged for them vanish). A wave (128 rows) reads one stage as 1 or 2 KiB, contiguous.
constexpr int kScaleRows = 128;
constexpr int fp4_scale_stage_bytes(bool asym) { return 32 * 4 * 8 * (asym ? 2 : 1); }

static int64_t fp4_packed_scale_bytes(bool asym, int64_t rows, int64_t K) {
  return (round_up(rows, kPanelRows) / kScaleRows) * ((K + 255) / 256) * fp4_scale_stage_bytes(asym);
}

size_t fp4_path_workspace_bytes(bool asym, int64_t M, int64_t N, int64_t K, int64_t batch) {
  return (size_t)(batch * (fp4_packed_scale_bytes(asym, M, K) + fp4_packed_scale_bytes(asym, N, K)));
}

// One operand of the re-layout: canonical scales [batch][R][G][SB] -> packed (Rp rows, a multiple of 128).
struct ScalePackJob {
  const uint8_t* scales;
  uint8_t* packed;
  int64_t R, Rp;
  int blocks;  // workgroups of this operand per batch entry: (Rp / 128) * ceil(stages / 16)
};

// grid: (jobA.blocks + jobB.blocks, 1, batch); block 256. A workgroup re-lays 128 rows x 16 stages: it reads the
// 128 * SB bytes those stages occupy in each of its rows (whole cache lines, 4 bytes per thread and load), turns them
// through LDS and writes 16 stages of packed scales, contiguous. SB: bytes per group (1 symmetric, 2 asymmetric).
template <int SB>
__global__ __launch_bounds__(256) void scale_pack_kernel(ScalePackJob ja, ScalePackJob jb, int64_t G, int nstages) {
  constexpr int kRowWords = 16 * 8 * SB / 4;  // 32-bit words of 16 stages of one row
  __shared__ uint32_t turn[kScaleRows][kRowWords + 1];
  const bool second = (int)blockIdx.x >= ja.blocks;
  const ScalePackJob& job = second ? jb : ja;
  const int blk = (int)blockIdx.x - (second ? ja.blocks : 0);
  const int chunks = (nstages + 15) / 16;
  const int64_t q = blk / chunks, b = blockIdx.z;
  const int st0 = (blk % chunks) * 16;
  const int64_t row_words = G * SB / 4;  // (scale rows are whole words: G is a multiple of 4)
  const uint32_t* src = reinterpret_cast<const uint32_t*>(job.scales) + b * job.R * row_words;
  for (int idx = threadIdx.x; idx < kScaleRows * kRowWords; idx += 256) {
    const int r = idx / kRowWords, w = idx % kRowWords;
    const int64_t row = q * kScaleRows + r, word = (int64_t)st0 * (8 * SB / 4) + w;
    turn[r][w] = (row < job.R && word < row_words) ? src[row * row_words + word] : 0u;
  }
  __syncthreads();
  // packed: [q][stage][r 32][i 4][8 * SB bytes]; one 8 * SB-byte entry = 2 * SB words
  constexpr int kEntryWords = 2 * SB, kStageWords = 32 * 4 * kEntryWords;
  uint32_t* dst = reinterpret_cast<uint32_t*>(job.packed) + ((b * (job.Rp / kScaleRows) + q) * nstages + st0) * kStageWords;
  const int stages_here = nstages - st0 < 16 ? nstages - st0 : 16;
  for (int idx = threadIdx.x; idx < stages_here * kStageWords; idx += 256) {
    const int st = idx / kStageWords, e = (idx % kStageWords) / kEntryWords, w = idx % kEntryWords;
    const int r = e >> 2, i = e & 3;
    dst[idx] = turn[i * 32 + r][st * kEntryWords + w];
  }
}

// One stage = a K slice of 256: 128 bytes = one whole cache line of every code row (a compute unit's vector cache
// tracks a limited number of line requests, so fetching half lines would halve what it can pull from the L2).
// LDS: two stage buffers of 64 KiB (A rows then B rows, 128 bytes per row). A stage is 4 k-steps x FM steps of FN
// MFMAs; fragments are read two steps (A) / one k-step (B) ahead. The next stage is fetched into the other buffer
// during the first half of a stage. The single barrier of a stage comes after step 13 of 16: by then every wave has
// its last fragments of the current buffer and the next stage has landed; the two steps after it read ahead into the
// next buffer.
// GLU: the gated-activation epilogue of store_glu_tiles() (gemm_common.h); C is then the BF16 output [M][ldc].
template <int WM, int WN, int FM, int FN, bool ASYM, bool GLU = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_fp4_kernel(const uint8_t* __restrict__ Ac,
                                                                const uint8_t* __restrict__ Asp,
                                                                const uint8_t* __restrict__ Bc,
                                                                const uint8_t* __restrict__ Bsp, float* __restrict__ C,
                                                                int64_t M, int64_t N, int64_t K, int64_t ldc,
                                                                int tiles_m, int tiles_n, int super_m) {
  using Cfg = TileCfg<WM, WN, FM, FN>;
  constexpr int kWaves = Cfg::kWaves, kTileM = Cfg::kTileM, kTileN = Cfg::kTileN;
  constexpr int kUnitsA = kTileM / 8, kUnitsB = kTileN / 8;  // direct-to-LDS loads (8 rows x 128 bytes) per stage
  constexpr int kLoads = (kUnitsA + kUnitsB) / kWaves;       // per wave and stage
  constexpr int kBytesA = kTileM * 128, kBytesB = kTileN * 128;
  static_assert(kUnitsA % kWaves == 0 && kUnitsB % kWaves == 0 && kWaves % 2 == 0 && FM == 4 && FN == 4 &&
                    kLoads == 16,
                "the issue schedule below is written for 2 x 2 waves of 4 x 4 MFMA tiles");
  // separate arrays per buffer and operand: the compiler can then tell that a direct-to-LDS load into one cannot
  // touch what a fragment read of another returns, and does not serialise them
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kBytesA];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsB0[kBytesB];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kBytesA];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsB1[kBytesB];

#define lds0_A ldsA0
#define lds0_B ldsB0
#define lds1_A ldsA1
#define lds1_B ldsB1
  typedef __attribute__((address_space(3))) const uint8_t* lds_cptr_t;
#define rd0_A ((lds_cptr_t)ldsA0)
#define rd0_B ((lds_cptr_t)ldsB0)
#define rd1_A ((lds_cptr_t)ldsA1)
#define rd1_B ((lds_cptr_t)ldsB1)
#define AMX_LDS_READ(P, OFF) (*reinterpret_cast<const __attribute__((address_space(3))) u32x4*>((P) + (OFF)))

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int64_t b = blockIdx.z;
  int tm, tn;
  if (!tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, super_m, tm, tn)) return;  // uniform, before any barrier

  const int row_bytes = (int)(K >> 1);                         // codes per row
  const int nstages_all = (int)((K + 255) >> 8);               // stages of the packed scales (the last may be half)
  const int rows_a = (int)(M - (int64_t)tm * kTileM < kTileM ? M - (int64_t)tm * kTileM : kTileM);
  const int rows_b = (int)(N - (int64_t)tn * kTileN < kTileN ? N - (int64_t)tn * kTileN : kTileN);

  // Raw buffer descriptors over this tile's rows: anything past the last valid row reads as zero. A zero scale byte
  // is 2^-127, so rows beyond M / N contribute products that vanish (and their outputs are never stored).
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Ac + (b * M + (int64_t)tm * kTileM) * row_bytes), 0, rows_a * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bc + (b * N + (int64_t)tn * kTileN) * row_bytes), 0, rows_b * row_bytes, 0x00020000);
  // packed scales of this wave's 128 rows of either operand: [stage][32 rows][4 row blocks][8 groups] entries
  constexpr int kStageScaleBytes = fp4_scale_stage_bytes(ASYM);
  const int64_t groups_m = (int64_t)tiles_m * (kTileM / kScaleRows), groups_n = (int64_t)tiles_n * (kTileN / kScaleRows);
  const __amdgpu_buffer_rsrc_t Asr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Asp + ((b * groups_m + (int64_t)tm * (kTileM / kScaleRows) + wm) * nstages_all) *
                                     kStageScaleBytes),
      0, nstages_all * kStageScaleBytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bsp + ((b * groups_n + (int64_t)tn * (kTileN / kScaleRows) + wn) * nstages_all) *
                                     kStageScaleBytes),
      0, nstages_all * kStageScaleBytes, 0x00020000);

  // Staging geometry. One direct-to-LDS load moves 8 rows x 128 bytes (8 lanes per row). Its LDS image is [8 rows]
  // [8 chunks of 16 bytes]; the chunk a lane fetches is permuted by the row, chunk = slot ^ ((row >> 1) & 7), so that
  // the fragment reads below (32 consecutive rows, one chunk each) fall on 16 distinct 16-byte bank groups per 16
  // lanes. Load unit u = wave + kWaves * L covers tile rows 8u .. 8u+7, so (row >> 1) & 7 = 4 * (u & 1) + row_in_unit
  // / 2, and u & 1 = wave & 1 for every unit of a wave.
  const int kb = lane >> 5;  // K block (of 32 codes) of this lane inside a 64-wide k-step
  const int gather_off = (lane >> 3) * row_bytes + (((lane & 7) ^ (4 * (wave & 1) + ((lane >> 4) & 3))) << 4);
  const int sgather_off = (lane & 31) * (kStageScaleBytes / 32);  // this lane's row inside a stage of packed scales
  // fragment read offset inside a row block (32 rows x 128 bytes) for k-step ks: chunk 2 ks + kb of row lane % 32
  const int rr = lane & 31;
  const int frag_row = rr * 128, frag_swz = (rr >> 1) & 7;
#define AMX_FRAG_OFF(KS) (frag_row + (((2 * (KS) + kb) ^ frag_swz) << 4))

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Load L of this wave for stage ST: L < kUnitsA / kWaves: unit u = wave + kWaves * L of operand A, otherwise unit
  // wave + kWaves * (L - kUnitsA / kWaves) of B. Lands at u KiB of the buffer DST##A / DST##B. Past the end of K the
  // stage index is clamped by the caller: the data lands where nobody reads it.
#define AMX_ISSUE_LOAD(L, ST, DST)                                                                              \
  {                                                                                                             \
    if ((L) < kUnitsA / kWaves) {                                                                               \
      const int u_ = wave + kWaves * (L);                                                                       \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)(DST##A + u_ * 1024), 16, gather_off,             \
                                               u_ * 8 * row_bytes + (ST) * 128, 0, 0);                          \
    } else {                                                                                                    \
      const int u_ = wave + kWaves * ((L) - kUnitsA / kWaves);                                                  \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)(DST##B + u_ * 1024), 16, gather_off,             \
                                               u_ * 8 * row_bytes + (ST) * 128, 0, 0);                          \
    }                                                                                                           \
  }

  // Scale words of one stage (8 groups of this lane's row), per row block: symmetric = 8 bytes (one per group),
  // asymmetric = 16 bytes ((pos, neg) per group); the four row blocks of a wave lie side by side in the packed array,
  // so a lane fetches them with two (four) 16-byte loads. Two register sets alternate between stages.
  static_assert(FM == 4 && FN == 4, "the packed scales hold four row blocks per wave");
  typedef uint32_t sword_t __attribute__((ext_vector_type(ASYM ? 4 : 2)));
  sword_t sa[2][FM], sb[2][FN];
  // part P (0, 1) of the scale fetch of one operand: the row blocks 2 P and 2 P + 1
#define AMX_LOAD_SCALES_PART(DSTV, RSRC, ST, P)                                                                     \
  {                                                                                                                 \
    if constexpr (ASYM) {                                                                                           \
      _Pragma("unroll") for (int i = 2 * (P); i < 2 * (P) + 2; ++i) DSTV[i] = __builtin_bit_cast(                   \
          sword_t, __builtin_amdgcn_raw_buffer_load_b128(RSRC, sgather_off + i * 16, (ST) * kStageScaleBytes, 0));  \
    } else {                                                                                                        \
      const u32x4 w_ = __builtin_bit_cast(                                                                          \
          u32x4, __builtin_amdgcn_raw_buffer_load_b128(RSRC, sgather_off + (P) * 16, (ST) * kStageScaleBytes, 0));  \
      DSTV[2 * (P)][0] = w_.x, DSTV[2 * (P)][1] = w_.y, DSTV[2 * (P) + 1][0] = w_.z, DSTV[2 * (P) + 1][1] = w_.w;   \
    }                                                                                                               \
  }
#define AMX_LOAD_SCALES(SET, ST)                  \
  {                                               \
    AMX_LOAD_SCALES_PART(sa[SET], Asr, ST, 0);    \
    AMX_LOAD_SCALES_PART(sa[SET], Asr, ST, 1);    \
    AMX_LOAD_SCALES_PART(sb[SET], Bsr, ST, 0);    \
    AMX_LOAD_SCALES_PART(sb[SET], Bsr, ST, 1);    \
  }
  constexpr int kScaleLoads = ASYM ? 8 : 4;  // vector loads of one AMX_LOAD_SCALES

  const int nfull = (int)(K >> 8);  // whole stages; K % 256 == 128 leaves half a stage for the end
  u32x4 aR[4], bR[2][FN];
  const int baseA = (wm * FM) * 4096;
  const int baseB = (wn * FN) * 4096;
  // The MFMAs of step (KS4, I) of a stage whose scale words are in set SET; k-step KS4 = 0..3 covers groups 2 KS4 and
  // 2 KS4 + 1 of the stage. Scale byte selection:
  // symmetric: word KS4 / 2 = bytes of 4 groups, shifted by 8*kb; the k-step uses byte OPS = 2 * (KS4 % 2) (opsel);
  // asymmetric: word KS4 = bytes (p0 n0 p1 n1) of the k-step, shifted by 16*kb; pos = byte 0, neg = byte 1.
#define AMX_MMA1(SET, KS4, I, J, OPS)                                                                                \
  {                                                                                                                  \
    if constexpr (!ASYM) {                                                                                           \
      const int sav = (int)(sa[SET][I][(KS4) >> 1] >> (8 * kb));                                                     \
      const int sbv = (int)(sb[SET][J][(KS4) >> 1] >> (8 * kb));                                                     \
      acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(aR[((KS4) * FM + (I)) & 3]),            \
                                                                  as_operand(bR[(KS4) & 1][J]), acc[I][J], 4, 4, OPS, \
                                                                  sav, OPS, sbv);                                    \
    } else {                                                                                                         \
      const int sav = (int)(sa[SET][I][KS4] >> (16 * kb));                                                           \
      const int sbv = (int)(sb[SET][J][KS4] >> (16 * kb));                                                           \
      const u32x4 araw = aR[((KS4) * FM + (I)) & 3];                                                                 \
      const i32x8 ap = as_operand(sign_class4<false>(araw)), an = as_operand(sign_class4<true>(araw));              \
      const i32x8 bp = as_operand(sign_class4<false>(bR[(KS4) & 1][J])),                                             \
                  bn = as_operand(sign_class4<true>(bR[(KS4) & 1][J]));                                              \
      acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ap, bp, acc[I][J], 4, 4, 0, sav, 0, sbv);          \
      acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ap, bn, acc[I][J], 4, 4, 0, sav, 1, sbv);          \
      acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(an, bp, acc[I][J], 4, 4, 1, sav, 0, sbv);          \
      acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(an, bn, acc[I][J], 4, 4, 1, sav, 1, sbv);          \
    }                                                                                                                \
  }
#define AMX_MMA(SET, KS4, I, OPS) \
  { _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_) AMX_MMA1(SET, KS4, I, j_, OPS); }
  /* (the scale-byte selector must be a literal: OPS = 2 * (ks % 2)) */
#define AMX_SLOT_MMA(SET, KS4, I, J) \
  { if (((KS4) & 1) == 0) AMX_MMA1(SET, KS4, I, J, 0) else AMX_MMA1(SET, KS4, I, J, 2); }

  // Stage S (scale words in set SET; CUR / NXT: the arrays of this and of the next stage as load destinations; RC /
  // RN: their read pointers). Step t = 4 ks + i multiplies A row block i with the four B row blocks of k-step ks: four
  // slots of one MFMA (asymmetric: four) each. A wave issues in order and has its SIMD to itself, so whatever stands
  // between two MFMAs must fit into the 32 cycles the first one occupies the matrix pipe: everything else a step does
  // is therefore dealt out over its slots, at most two memory instructions in front of any MFMA (with all of a
  // step's loads and fragment reads in front of its first MFMA every direct-to-LDS load cost the pipe about 58
  // idle cycles, a third of the main loop):
  //   - slot 0: the A fragment of step t + 2 (read ahead; the last two steps read into the next stage's arrays);
  //   - slots 1, 2 of the steps i = 0, 1 (i = 2, 3 in the last k-step, after the barrier, from the next stage's
  //     arrays): the four B fragments of the next k-step;
  //   - the 16 direct-to-LDS loads of stage S + 1 are spread over twelve steps: the arrays they go to are free once
  //     the barrier of stage S - 1 has passed, so four are issued in the last two steps of stage S - 1 (as loads 0..3
  //     of stage S + 2 into CUR here), four in steps 0 and 1 and eight in steps 2..9, in the slots without a B read;
  //   - steps 10 and 11: the scale words of stage S + 1 (A's, then B's) into the other register set;
  //   - after step 13: wait for the direct-to-LDS loads (not for the scale words, which are younger) and for this
  //     wave's fragment reads, barrier: every wave has its last fragments of CUR and stage S + 1 has landed.
#define AMX_DMA(T, WHICH, CUR, NXT)                                                                                      \
  {                                                                                                               \
    if ((T) < 2) AMX_ISSUE_LOAD(4 + 2 * (T) + (WHICH), next_, NXT)                                                \
    else if ((T) < 10) AMX_ISSUE_LOAD(6 + (T), next_, NXT)                                                        \
    else AMX_ISSUE_LOAD(2 * ((T) - kLast - 1) + (WHICH), next2_, CUR)                                             \
  }
#define AMX_STAGE(S, SET, CUR, NXT, RC, RN)                                                                        \
  {                                                                                                               \
    const int next_ = (S) + 1 < nfull ? (S) + 1 : nfull - 1;                                                      \
    const int next2_ = (S) + 2 < nfull ? (S) + 2 : nfull - 1;                                                     \
    constexpr int kLast = 4 * FM - 3; /* the step followed by the barrier */                                      \
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                                            \
      _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                            \
        const int t = ks * FM + i;                                                                                \
        const bool b_reads = ks < 3 ? i < 2 : i >= 2;                                                             \
        const int jj = ks < 3 ? 2 * i : 2 * (i - 2);                                                              \
        const int dma = t < 2 ? 2 : t < 10 ? 1 : t > kLast ? 2 : 0; /* direct-to-LDS loads of this step */        \
        /* slot 0 */                                                                                              \
        {                                                                                                         \
          const int t2 = t + 2, ks2 = t2 / FM, i2 = t2 % FM;                                                      \
          if (ks2 < 4)                                                                                            \
            aR[t2 & 3] = AMX_LDS_READ(RC##A, baseA + i2 * 4096 + AMX_FRAG_OFF(ks2 & 3));                          \
          else                                                                                                    \
            aR[t2 & 3] = AMX_LDS_READ(RN##A, baseA + i2 * 4096 + AMX_FRAG_OFF(0));                                \
        }                                                                                                         \
        if (b_reads && dma == 2) AMX_DMA(t, 1, CUR, NXT);                                                                   \
        AMX_SLOT_MMA(SET, ks, i, 0);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        /* slot 1 */                                                                                              \
        if (b_reads) {                                                                                            \
          if (ks < 3) bR[(ks + 1) & 1][jj] = AMX_LDS_READ(RC##B, baseB + jj * 4096 + AMX_FRAG_OFF(ks + 1));       \
          else bR[0][jj] = AMX_LDS_READ(RN##B, baseB + jj * 4096 + AMX_FRAG_OFF(0));                              \
        } else if (dma >= 1) {                                                                                    \
          AMX_DMA(t, 0, CUR, NXT);                                                                                          \
        } else if (t == 10) {                                                                                     \
          AMX_LOAD_SCALES_PART(sa[(SET) ^ 1], Asr, next_, 0);                                                     \
        } else if (t == 11) {                                                                                     \
          AMX_LOAD_SCALES_PART(sb[(SET) ^ 1], Bsr, next_, 0);                                                     \
        }                                                                                                         \
        AMX_SLOT_MMA(SET, ks, i, 1);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        /* slot 2 */                                                                                              \
        if (b_reads) {                                                                                            \
          if (ks < 3) bR[(ks + 1) & 1][jj + 1] = AMX_LDS_READ(RC##B, baseB + (jj + 1) * 4096 + AMX_FRAG_OFF(ks + 1)); \
          else bR[0][jj + 1] = AMX_LDS_READ(RN##B, baseB + (jj + 1) * 4096 + AMX_FRAG_OFF(0));                    \
        } else if (t == 10) {                                                                                     \
          AMX_LOAD_SCALES_PART(sa[(SET) ^ 1], Asr, next_, 1);                                                     \
        } else if (t == 11) {                                                                                     \
          AMX_LOAD_SCALES_PART(sb[(SET) ^ 1], Bsr, next_, 1);                                                     \
        }                                                                                                         \
        AMX_SLOT_MMA(SET, ks, i, 2);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        /* slot 3 */                                                                                              \
        if (b_reads && dma >= 1) AMX_DMA(t, 0, CUR, NXT);                                                                   \
        AMX_SLOT_MMA(SET, ks, i, 3);                                                                              \
        if (t == kLast) {                                                                                         \
          /* vmcnt(kScaleLoads) lgkmcnt(0): all but the youngest vector loads, which are the scale words */       \
          __builtin_amdgcn_s_waitcnt(0x0070 | kScaleLoads);                                                       \
          AMX_BARRIER();                                                                                          \
        }                                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
      }                                                                                                           \
    }                                                                                                             \
  }

  if (nfull > 0) {
    // prologue: stage 0
#pragma unroll
    for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 0, lds0_);
    AMX_LOAD_SCALES(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0070);  // everything
    AMX_BARRIER();
    aR[0] = AMX_LDS_READ(rd0_A, baseA + AMX_FRAG_OFF(0));
    aR[1] = AMX_LDS_READ(rd0_A, baseA + 4096 + AMX_FRAG_OFF(0));
#pragma unroll
    for (int j = 0; j < FN; ++j)
      bR[0][j] = AMX_LDS_READ(rd0_B, baseB + j * 4096 + AMX_FRAG_OFF(0));
    {  // the first four loads of stage 1 (the stages issue loads 4..15 of their successor themselves)
      const int st1_ = nfull > 1 ? 1 : 0;
#pragma unroll
      for (int l = 0; l < 4; ++l) AMX_ISSUE_LOAD(l, st1_, lds1_);
    }
    int s = 0;
    for (; s + 2 <= nfull; s += 2) {
      AMX_STAGE(s, 0, lds0_, lds1_, rd0_, rd1_);
      AMX_STAGE(s + 1, 1, lds1_, lds0_, rd1_, rd0_);
    }
    if (s < nfull) AMX_STAGE(s, 0, lds0_, lds1_, rd0_, rd1_);
    __builtin_amdgcn_s_waitcnt(0x0070);  // this wave's last (unused) prefetches have landed, its reads are done
    AMX_BARRIER();                       // ... and everybody else's: LDS is free
  }
  if (K & 255) {
    // The last 128 of K, not pipelined (once per tile): the loads fetch whole lines again, the second half of which
    // belongs to the next row (or reads as zero past the tile's last row) and is not used.
#pragma unroll
    for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, nfull, lds0_);
    AMX_LOAD_SCALES(0, nfull);
    __builtin_amdgcn_s_waitcnt(0x0070);
    AMX_BARRIER();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int j = 0; j < FN; ++j)
        bR[ks & 1][j] = AMX_LDS_READ(rd0_B, baseB + j * 4096 + AMX_FRAG_OFF(ks));
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        aR[(ks * FM + i) & 3] = AMX_LDS_READ(rd0_A, baseA + i * 4096 + AMX_FRAG_OFF(ks));
        if (ks == 0) AMX_MMA(0, ks, i, 0) else AMX_MMA(0, ks, i, 2);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_DMA
#undef AMX_SLOT_MMA
#undef AMX_MMA
#undef AMX_MMA1
#undef AMX_LOAD_SCALES
#undef AMX_LOAD_SCALES_PART
#undef AMX_ISSUE_LOAD
#undef AMX_FRAG_OFF
#undef AMX_LDS_READ
#undef lds0_A
#undef lds0_B
#undef lds1_A
#undef lds1_B

  if constexpr (GLU) {
    // every wave is past its last fragment read: the operand stages become the waves' transposition space
    static_assert(kWaves <= 4 && glu_stage_bytes<FM, FN>() <= kBytesA && glu_stage_bytes<FM, FN>() <= kBytesB,
                  "stage too small");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    AMX_BARRIER();
    const int w = wm * WN + wn;
    uint8_t* stage = w == 0 ? ldsA0 : w == 1 ? ldsB0 : w == 2 ? ldsA1 : ldsB1;
    store_glu_tiles<FM, FN>(acc, stage, reinterpret_cast<uint16_t*>(C) + b * M * ldc, M, N >> 1, ldc,
                            (int64_t)tm * kTileM + wm * FM * 32, (int64_t)tn * kTileN + wn * FN * 32);
  } else
    store_c_tiles<FM, FN>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * kTileM + wm * FM * 32,
                          (int64_t)tn * kTileN + wn * FN * 32);
}

bool fp4_path_supported(int64_t M, int64_t N, int64_t K) {
  // K in whole stages; per-tile byte offsets (256 rows x K/2 bytes, 256 rows x K/16 bytes) must fit the 32-bit
  // buffer offsets
  return K % 128 == 0 && K <= (1 << 22) && M > 0 && N > 0;
}

template <bool ASYM>
static hipError_t launch_fp4(int64_t M, int64_t N, int64_t K, const uint8_t* Ac, const uint8_t* As, const uint8_t* Bc,
                             const uint8_t* Bs, float* C, int64_t ldc, int64_t batch, void* workspace, hipStream_t s,
                             const KernelTimer& timer, bool glu) {
  using Cfg = TileCfg<2, 2, 4, 4>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  // the scale bytes of both operands, re-laid in the order the waves fetch them
  constexpr int SB = ASYM ? 2 : 1;
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows), G = K >> 5;
  const int nstages = (int)((K + 255) / 256);
  uint8_t* Asp = reinterpret_cast<uint8_t*>(workspace);
  uint8_t* Bsp = Asp + batch * fp4_packed_scale_bytes(ASYM, M, K);
  const int chunks = (nstages + 15) / 16;
  const ScalePackJob ja = {As, Asp, M, Mp, (int)(Mp / kScaleRows) * chunks};
  const ScalePackJob jb = {Bs, Bsp, N, Np, (int)(Np / kScaleRows) * chunks};
  hipLaunchKernelGGL((scale_pack_kernel<SB>), dim3((unsigned)(ja.blocks + jb.blocks), 1, (unsigned)batch), dim3(256),
                     0, s, ja, jb, G, nstages);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  if (glu)
    hipLaunchKernelGGL((gemm_fp4_kernel<2, 2, 4, 4, ASYM, true>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads),
                       0, s, Ac, Asp, Bc, Bsp, C, M, N, K, ldc, tiles_m, tiles_n, super_m);
  else
    hipLaunchKernelGGL((gemm_fp4_kernel<2, 2, 4, 4, ASYM>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s,
                       Ac, Asp, Bc, Bsp, C, M, N, K, ldc, tiles_m, tiles_n, super_m);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

hipError_t launch_gemm_fp4_path(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                int64_t ldc, int64_t batch, void* workspace, hipStream_t s, const KernelTimer& timer,
                                bool glu) {
  return asym ? launch_fp4<true>(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace, s, timer, glu)
              : launch_fp4<false>(M, N, K, A_codes, A_scales, B_codes, B_scales, C, ldc, batch, workspace, s, timer, glu);
}

}  // namespace amx
