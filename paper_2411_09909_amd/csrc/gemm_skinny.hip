// Fully quantized GEMM (Sec. 4.3) for a small number of rows on the A side (M <= 256: a few tokens against a weight
// matrix). Such a product is bound by reading the weights, and the point of 4-bit weights is that they are a quarter
// of the BF16 bytes, so this kernel reads the packed codes and scales of B straight from memory, dequantizes them in
// registers to exact 16-bit floats (element * scale has at most 6 significant bits) and feeds the 16-bit MFMA; only
// the small A operand goes through a panel (expand_kernel). No operand of B is ever written back.
// The dequantization is the kernel's bound (vector instructions per MFMA), so it uses packed 16-bit arithmetic where
// the scale format allows it:
//   FP8-E5M2 scales: FP16 operands biased by 2^-3 (every element * scale * 2^-3 lies in [2^-20, 43008] and has at most
//     5 significant bits: an FP16 number, subnormals included). The scale byte is the upper byte of an FP16, so a pair
//     of scales is one byte permute; v_cvt_scalef32_pk_f16_fp4 turns two codes into two FP16 elements / 8, a packed
//     arithmetic shift of the sign bits selects the scale pair of each sign class and one packed multiply finishes.
//     A comes from an FP16 panel with the same bias and the result is multiplied by 2^6.
//   power-of-two scales: v_cvt_scalef32_pk_bf16_fp4 applies the scale itself (two codes -> two BF16 per instruction);
//     the asymmetric format converts with both scales and selects per sign.
//   FP8-E4M3 scales: FP32 conversion, multiply, truncate to BF16.
//
// Work split: one workgroup = 8 (4 with more than four row tiles) waves = neighbouring tiles of 32 columns of C (32
// rows of B each) over one outer K slice; with a single row tile (M <= 32) two waves share a column tile and take
// alternate K blocks. K is walked in blocks of 256. The workgroup brings the A operand into LDS
// once, by direct-to-LDS loads, in stages of half a block (a whole block per wave of a column tile for one or two row
// tiles), double buffered.
// Each lane owns half a B row's block: row lane % 32 of its wave's tile, groups 4 h .. 4 h + 3 for lane half
// h = lane / 32, i.e. 64 contiguous bytes of codes (the two halves of a wave share every 128-byte cache line, fetched
// once) and 4 scale entries, loaded one block ahead. It then runs the block's 16 k-steps from registers: k-step s
// multiplies the 8 codes s % 4 of the lane's group s / 4. The k order this gives a block (half h of k-step s = the 8
// elements s % 4 of group 4 h + s / 4) is not the natural one; the A panel is written in the same order
// (expand_kernel<HALF_LINE>), and a sum over k does not depend on it. With more than one outer slice the partial tiles
// go to the workspace and a second kernel adds them in a fixed order (no atomics: results are reproducible).

#include "dequant_regs.h"
#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
// scale arrays are only 4-byte aligned by contract: vectors of them are loaded through under-aligned types
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));

// The scale pair of a lane's group GI (0 .. 3) from its scale registers (asymmetric: bytes pos, neg of the four
// groups in S[0], S[1]; symmetric: the four bytes of S[0]), in the form dequant_word() takes.
template <int SCALE_KIND, bool ASYM, int GI>
__device__ __forceinline__ void skinny_scales(const uint32_t (&S)[2], uint32_t& s_pos, uint32_t& s_neg) {
  constexpr uint32_t bp = ASYM ? 2 * (GI & 1) : GI, bn = ASYM ? bp + 1 : bp;
  const uint32_t reg = S[ASYM ? GI >> 1 : 0];
  if constexpr (SCALE_KIND == kScaleE5M2) {
    // byte -> (byte << 8) in both halves; the cast never sets a scale's sign bit and it is ignored
    s_pos = __builtin_amdgcn_perm(0u, reg, (bp << 24) | (0x0Cu << 16) | (bp << 8) | 0x0Cu) & 0x7F007F00u;
    s_neg = ASYM ? __builtin_amdgcn_perm(0u, reg, (bn << 24) | (0x0Cu << 16) | (bn << 8) | 0x0Cu) & 0x7F007F00u : s_pos;
  } else if constexpr (SCALE_KIND == kScaleE8M0Floor) {
    s_pos = ((reg >> (8 * bp)) & 255u) << 23;
    s_neg = ASYM ? ((reg >> (8 * bn)) & 255u) << 23 : s_pos;
  } else {
    s_pos = f2u(scale_value<SCALE_KIND>((reg >> (8 * bp)) & 255u));
    s_neg = ASYM ? f2u(scale_value<SCALE_KIND>((reg >> (8 * bn)) & 255u)) : s_pos;
  }
}

constexpr int kSkinnyMaxM = 256;    // at most eight 32-row MFMA tiles
constexpr int kSkinnyBlockK = 256;  // K block: 128 bytes of codes per row
// Waves per workgroup = 32-column tiles of C it covers: every workgroup reads the whole A slice, so wider workgroups
// mean less A traffic; with more than four row tiles a wave needs more than the 256 registers an 8-wave workgroup
// leaves it.
constexpr int skinny_waves(int row_tiles) { return row_tiles <= 4 ? 8 : 4; }
// K phases inside a workgroup. With a single row tile a wave holds little (16 accumulators, one block of codes) and
// two workgroups fit a compute unit: there, two waves share each 32-column tile and take alternate K blocks, and
// their sums are added through LDS at the end (a fixed order, no further traffic to memory). The same number of
// waves then needs half the outer K slices (measured, 32 x 28672 x 8192: 43.1 -> 40.2 us for the call, with one
// slice and no partial tiles instead of two; four phases in workgroups of 16 waves were no faster, and with two row
// tiles the same split gains on 64 x 28672 x 8192, 56.5 -> 53.2 us, what it loses on smaller problems).
constexpr int skinny_k_phases(int row_tiles) { return row_tiles == 1 ? 2 : 1; }
// columns of C a workgroup covers
constexpr int skinny_cols(int row_tiles) { return 32 * skinny_waves(row_tiles) / skinny_k_phases(row_tiles); }

// Outer K slices for a problem with `groups` workgroups per slice, nblk K blocks and Mp padded rows. A workgroup's
// time is its number of K blocks; the chip runs 256 workgroups at a time (a second resident workgroup per CU mostly
// waits for the same memory system), so a launch takes ceil(workgroups / 256) * blocks_per_slice block times, plus the
// partial tiles every further slice writes and the reduction reads (16 Mp / K of the bytes of B per slice). The
// cheapest count of at most 16 wins, the smaller one on ties. Returns the number of slices and sets the blocks per
// slice; every slice has at least one block ((slices - 1) * blocks_per_slice < nblk).
// forced > 0 (a caller's tuning option) takes the place of the model's count.
static int skinny_outer_slices(int64_t groups, int64_t nblk, int64_t Mp, int forced, int& blocks_per_slice) {
  const double b_time = (double)(groups * nblk) / 256.0, partial = 16.0 * (double)Mp / (double)(nblk * kSkinnyBlockK);
  int64_t best = 1;
  double best_cost = 1e300;
  for (int64_t want = 1; want <= 16 && want <= nblk; ++want) {
    const int64_t bps = (nblk + want - 1) / want, slices = (nblk + bps - 1) / bps;
    const double rounds = (double)((groups * slices + 255) / 256);
    const double cost = rounds * (double)bps + (slices > 1 ? b_time * partial * (double)slices : 0.0);
    if (cost < best_cost - 1e-9) best_cost = cost, best = want;
  }
  if (forced > 0) best = forced < nblk ? forced : nblk;
  blocks_per_slice = (int)((nblk + best - 1) / best);
  return (int)((nblk + blocks_per_slice - 1) / blocks_per_slice);
}

// 32-row tiles the kernel is instantiated for: 1 .. 4, 6, 8 (A's panel and the partial tiles are padded to that)
static int skinny_row_tiles(int64_t M) {
  const int t = (int)((M + 31) / 32);
  return t <= 4 ? t : (t <= 6 ? 6 : 8);
}

// More than kSkinnyMaxM rows (single problems only) run as row chunks of kSkinnyMaxM, one launch each over all of B:
// up to kSkinnyMaxChunkedM rows against at least 2^27 weight elements that is still faster than expanding B to BF16
// and streaming the panel (measured on 28672 x 8192 weights: 512 rows 0.30 against 0.48 ms, 768 rows 0.45 against
// 0.49 ms; the second and third pass find the 132 MB of codes in the last-level cache).
constexpr int kSkinnyMaxChunkedM = 768;

bool skinny_path_supported(int64_t M, int64_t N, int64_t K, int64_t batch) {
  if (K % kSkinnyBlockK != 0 || N < 1 || M < 1) return false;
  return M <= kSkinnyMaxM || (batch == 1 && M <= kSkinnyMaxChunkedM && N * K >= (int64_t(1) << 27));
}

// padded rows of the A panel: full chunks of kSkinnyMaxM, the last one rounded up to its row tiles
static int64_t skinny_panel_rows(int64_t M) {
  const int64_t full = (M - 1) / kSkinnyMaxM;
  return full * kSkinnyMaxM + 32 * skinny_row_tiles(M - full * kSkinnyMaxM);
}

// bytes of partial tiles one chunk of `rows` rows needs (0 with a single slice)
static size_t skinny_partial_bytes(int64_t rows, int64_t N, int64_t K, int64_t batch, int forced_slices) {
  const int64_t Mp = 32 * skinny_row_tiles(rows), cols = skinny_cols(skinny_row_tiles(rows));
  int bps;
  const int slices = skinny_outer_slices((N + cols - 1) / cols * batch, K / kSkinnyBlockK, Mp, forced_slices, bps);
  return slices > 1 ? (size_t)(batch * slices * Mp * N * 4) : 0;
}

size_t skinny_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int forced_slices) {
  size_t bytes = (size_t)(batch * skinny_panel_rows(M) * K * 2);  // A panel
  bytes = (bytes + 255) / 256 * 256;
  size_t partial = 0;  // the chunks run one after the other and share the partial tiles' space
  for (int64_t r0 = 0; r0 < M; r0 += kSkinnyMaxM) {
    const size_t p = skinny_partial_bytes(M - r0 < kSkinnyMaxM ? M - r0 : kSkinnyMaxM, N, K, batch, forced_slices);
    partial = p > partial ? p : partial;
  }
  return bytes + partial;
}

// grid: (ceil(N / skinny_cols(MT)), outer slices, batch); block = skinny_waves(MT) waves.
// (B_codes, B_scales and out are deliberately not declared restrict: loads the compiler knows to be from memory nobody
// writes may be moved across the barriers, down to their first use, which undoes the prefetch.)
// out: C (ld_out = ldc) when gridDim.y == 1, else partials [batch][slice][MT * 32][N].
template <int SCALE_KIND, bool ASYM, int MT>
__global__ __launch_bounds__(64 * skinny_waves(MT)) void gemm_skinny_kernel(
    const uint16_t* __restrict__ Ap, const uint8_t* B_codes, const uint8_t* B_scales, float* out, int64_t M, int64_t N,
    int64_t K, int64_t ld_out, int64_t batch_stride_out, int64_t slice_stride_out, int blocks_per_slice) {
  // One step of the main loop multiplies one A stage: half a K block (8 k-steps of 16), or a whole one when there are
  // so few row tiles that half a block is too little work between two barriers to cover the latency of the loads
  // that fill the other stage.
  constexpr int kStageSteps = MT <= 2 ? 16 : 8;
  constexpr int kSkinnyWaves = skinny_waves(MT);
  constexpr int KP = skinny_k_phases(MT);               // waves per column tile; wave (tile ct, phase ph)
  constexpr int kSubFrags = MT * kStageSteps;           // A fragments of one K block (or half block) of a stage
  constexpr int kFragsPerHalf = kSubFrags * KP;         // A fragments of one stage: one block per phase
  static_assert(KP == 1 || kStageSteps == 16, "K phases take whole blocks");
  constexpr bool kF16 = SCALE_KIND == kScaleE5M2;       // FP16 operands biased by 2^-3 each, else BF16
  // two stages, separate arrays so that loads into one are known not to alias reads of the other
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kFragsPerHalf * kFragBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kFragsPerHalf * kFragBytes];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = lane >> 5;
  const int ct = wave / KP, ph = wave % KP;
  const int64_t b = blockIdx.z;
  const int64_t n = ((int64_t)blockIdx.x * (kSkinnyWaves / KP) + ct) * 32 + (lane & 31);
  const bool valid = n < N;
  const int64_t G = K >> 5, nblk = K / kSkinnyBlockK;
  constexpr int kScaleBytes = ASYM ? 2 : 1;

  const int64_t s_begin = (int64_t)blockIdx.y * blocks_per_slice;
  const int nb = (int)((s_begin + blocks_per_slice < nblk ? s_begin + blocks_per_slice : nblk) - s_begin);  // >= 1

  const int64_t row = valid ? b * N + n : 0;  // (rows past N read row 0 and are discarded)
  // lane half h owns groups 4 h .. 4 h + 3 of every block: 64 contiguous bytes of codes, 4 scale entries
  const uint8_t* codes_row = B_codes + row * (K >> 1) + s_begin * (kSkinnyBlockK / 2) + h * 64;
  const uint8_t* scales_row = B_scales + (row * G + s_begin * 8 + h * 4) * kScaleBytes;
  // A panel of this batch entry: [MT row blocks][K / 16 fragments][64 lanes][8 x 16 bit]; raw buffer, reads past the end
  // return zero
  const int kfrags = (int)(K >> 4);
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(Ap) + b * (int64_t)MT * kfrags * kFragBytes), 0,
      MT * kfrags * kFragBytes, 0x00020000);
  const int lane_off = lane * 16;
  const int a_off = lane_off + ph * kSubFrags * kFragBytes;  // this wave's block within a stage
  const int first_frag = (int)s_begin * (kSkinnyBlockK / 16);

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;

  // wave w brings fragments w, w + waves, .. of A stage block HB into stage DST. A stage block is KP consecutive
  // K blocks of this slice (one per phase; half a block or a whole one when KP is 1); fragment f of the stage =
  // block f / kSubFrags of them, row block (f % kSubFrags) / kStageSteps, k-step f % kStageSteps. Blocks past the
  // end of the slice (the last stage block of an odd count) are not loaded and not read.
#define AMX_SKINNY_LOAD_A(HB, DST)                                                                                 \
  _Pragma("unroll") for (int i_ = 0; i_ < kFragsPerHalf / kSkinnyWaves; ++i_) {                                    \
    const int f_ = wave + kSkinnyWaves * i_, sub_ = f_ / kSubFrags, r_ = f_ % kSubFrags;                           \
    if (KP == 1 || (HB) * KP + sub_ < nb)                                                                          \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                                    \
          Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,                                                  \
          ((r_ / kStageSteps) * kfrags + first_frag + ((HB) * KP + sub_) * kStageSteps + (r_ % kStageSteps)) *     \
              kFragBytes,                                                                                          \
          0, 0);                                                                                                   \
  }
  // this lane's half of its row's cache line of codes (4 groups) and the 4 scale entries of block I
#define AMX_SKINNY_LOAD_B(I, W, S)                                                                                 \
  {                                                                                                                \
    const u32x4* csrc_ = reinterpret_cast<const u32x4*>(codes_row + (int64_t)(I) * (kSkinnyBlockK / 2));           \
    W[0] = csrc_[0], W[1] = csrc_[1], W[2] = csrc_[2], W[3] = csrc_[3];                                            \
    if constexpr (ASYM) {                                                                                          \
      const u32x2_a4 t_ = *reinterpret_cast<const u32x2_a4*>(scales_row + (int64_t)(I) * 16);                      \
      S[0] = t_[0], S[1] = t_[1];                                                                                  \
    } else {                                                                                                       \
      S[0] = *reinterpret_cast<const uint32_t*>(scales_row + (int64_t)(I) * 8), S[1] = 0;                          \
    }                                                                                                              \
  }
  // The four k-steps of the lane's group GI (a literal: register arrays must not be indexed with a run-time value) of
  // one block: k-step 4 GI + t multiplies word t of the group; A fragments from stage SRC, B from the registers W / S
#define AMX_SKINNY_KSTEP(SRC, WORD, KF)                                                                            \
  {                                                                                                                \
    const u32x4 q = dequant_word<SCALE_KIND, ASYM>(WORD, s_pos, s_neg);                                            \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                                            \
      const bf16x8 a = *reinterpret_cast<const bf16x8*>((SRC) + (mt * kStageSteps + (KF)) * kFragBytes + a_off);   \
      if constexpr (kF16)                                                                                          \
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),                             \
                                                         __builtin_bit_cast(f16x8, q), acc[mt], 0, 0, 0);          \
      else                                                                                                         \
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, q), acc[mt], 0, 0, 0);     \
    }                                                                                                              \
  }
#define AMX_SKINNY_GROUP(SRC, W, S, GI)                                                                            \
  {                                                                                                                \
    uint32_t s_pos, s_neg;                                                                                         \
    skinny_scales<SCALE_KIND, ASYM, GI>(S, s_pos, s_neg);                                                          \
    constexpr int kf0 = ((GI) * 4) % kStageSteps; /* the group's first k-step within its stage */                  \
    AMX_SKINNY_KSTEP(SRC, W[GI][0], kf0)                                                                           \
    AMX_SKINNY_KSTEP(SRC, W[GI][1], kf0 + 1)                                                                       \
    AMX_SKINNY_KSTEP(SRC, W[GI][2], kf0 + 2)                                                                       \
    AMX_SKINNY_KSTEP(SRC, W[GI][3], kf0 + 3)                                                                       \
  }
#define AMX_SKINNY_HALF0(SRC, W, S) AMX_SKINNY_GROUP(SRC, W, S, 0) AMX_SKINNY_GROUP(SRC, W, S, 1)
#define AMX_SKINNY_HALF1(SRC, W, S) AMX_SKINNY_GROUP(SRC, W, S, 2) AMX_SKINNY_GROUP(SRC, W, S, 3)

  u32x4 w0[4], w1[4];
  uint32_t s0[2], s1[2];
  AMX_SKINNY_LOAD_A(0, ldsA0);
  // (a phase without a first block, in a slice of a single block, loads block 0 and does not use it)
  AMX_SKINNY_LOAD_B(ph < nb ? ph : 0, w0, s0);
  // The first block's registers are named as used here so that their loads complete in front of the loop: the
  // compiler may otherwise sink them to their first use inside it, where waiting for them means waiting for nearly
  // every load issued since (the next block's among them), in every iteration.
  asm volatile("" ::"v"(w0[0]), "v"(w0[1]), "v"(w0[2]), "v"(w0[3]), "v"(s0[0]), "v"(s0[1]));
  AMX_WAIT_VMCNT(0);
  AMX_BARRIER();
  if constexpr (kStageSteps == 16) {
    // Step i multiplies stage block i (this wave: K block i KP + ph of the slice) from stage i % 2 with the codes in
    // register set i % 2, while the loads of step i + 1 fill the other stage and the other register set; each step
    // ends with a wait and a barrier, after which the stage it read may be refilled. All conditions are uniform
    // over the wave, those around the barriers over the workgroup.
    const int steps = (nb + KP - 1) / KP;
    for (int i = 0; i < steps; i += 2) {
      if (i + 1 < steps) {
        AMX_SKINNY_LOAD_A(i + 1, ldsA1);
        if ((i + 1) * KP + ph < nb) AMX_SKINNY_LOAD_B((i + 1) * KP + ph, w1, s1);
      }
      if (i * KP + ph < nb) {
        AMX_SKINNY_HALF0(ldsA0, w0, s0);
        AMX_SKINNY_HALF1(ldsA0, w0, s0);
      }
      AMX_WAIT_VMCNT(0);
      AMX_BARRIER();
      if (i + 1 < steps) {
        if (i + 2 < steps) {
          AMX_SKINNY_LOAD_A(i + 2, ldsA0);
          if ((i + 2) * KP + ph < nb) AMX_SKINNY_LOAD_B((i + 2) * KP + ph, w0, s0);
        }
        if ((i + 1) * KP + ph < nb) {
          AMX_SKINNY_HALF0(ldsA1, w1, s1);
          AMX_SKINNY_HALF1(ldsA1, w1, s1);
        }
        AMX_WAIT_VMCNT(0);
        AMX_BARRIER();
      }
    }
  } else {
    // Block i: its first half is multiplied from stage 0, its second from stage 1, with the codes in register set
    // i % 2. Every step fetches what the next step needs (the other A stage; the next block's codes during a first
    // half) and ends with a wait and a barrier, after which the stage it read may be refilled. All conditions are
    // uniform.
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
  }
#undef AMX_SKINNY_HALF1
#undef AMX_SKINNY_HALF0
#undef AMX_SKINNY_GROUP
#undef AMX_SKINNY_KSTEP
#undef AMX_SKINNY_LOAD_B
#undef AMX_SKINNY_LOAD_A

  if constexpr (KP > 1) {
    // the phases' sums of a column tile, added in ascending phase order through the first stage's memory (every
    // wave is past the last barrier of the loop, nothing reads the stages any more)
    static_assert((KP - 1) * (kSkinnyWaves / KP) * MT * 16 * 64 * 4 <= kFragsPerHalf * kFragBytes, "stage too small");
    float* red = reinterpret_cast<float*>(ldsA0);
    if (ph != 0) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          red[((((ph - 1) * (kSkinnyWaves / KP) + ct) * MT + mt) * 16 + v) * 64 + lane] = acc[mt][v];
    }
    __syncthreads();
    if (ph != 0) return;
#pragma unroll
    for (int p = 1; p < KP; ++p)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          acc[mt][v] += red[((((p - 1) * (kSkinnyWaves / KP) + ct) * MT + mt) * 16 + v) * 64 + lane];
  }
  // register v of row tile mt is row 32 mt + 8 (v / 4) + 4 h + v % 4, column n
  if (!valid) return;
  float* dst = out + b * batch_stride_out + (int64_t)blockIdx.y * slice_stride_out + n;
  const int64_t row_limit = gridDim.y == 1 ? M : (int64_t)MT * 32;  // partial tiles keep their padded rows
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t r = mt * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
      if (r < row_limit) dst[r * ld_out] = kF16 ? acc[mt][v] * 64.0f : acc[mt][v];  // undo the two biases
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
  constexpr int kWaves = skinny_waves(MT), kCols = skinny_cols(MT);
  const dim3 grid((unsigned)((N + kCols - 1) / kCols), (unsigned)slices, (unsigned)batch);
  if (slices == 1) {
    hipLaunchKernelGGL((gemm_skinny_kernel<SK, ASYM, MT>), grid, dim3(64 * kWaves), 0, s, Ap, Bc, Bs, C, M, N, K, ldc,
                       M * ldc, (int64_t)0, blocks_per_slice);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((gemm_skinny_kernel<SK, ASYM, MT>), grid, dim3(64 * kWaves), 0, s, Ap, Bc, Bs, partial, M, N, K, N,
                     (int64_t)slices * Mp * N, Mp * N, blocks_per_slice);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)((M * N + 255) / 256), 1, (unsigned)batch), dim3(256), 0, s,
                     partial, C, M, N, Mp, ldc, slices);
  return hipGetLastError();
}

hipError_t launch_gemm_skinny_path(int scale_kind, bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                   const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                   int64_t ldc, int64_t batch, void* workspace, int forced_slices, hipStream_t s,
                                   const KernelTimer& timer) {
  if (!skinny_path_supported(M, N, K, batch)) return hipErrorInvalidValue;
  const int64_t Mp_all = skinny_panel_rows(M);
  uint16_t* Ap = reinterpret_cast<uint16_t*>(workspace);
  const size_t panel_bytes = ((size_t)(batch * Mp_all * K * 2) + 255) / 256 * 256;
  float* partial = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(workspace) + panel_bytes);
  hipError_t e = launch_expand_half_line(scale_kind, asym, A_codes, A_scales, M, K, Mp_all, batch, Ap, s);
  if (e != hipSuccess) return e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  // E8M0 floor and round share the byte encoding
  const int sk = scale_kind == kScaleE8M0Round ? kScaleE8M0Floor : scale_kind;
  // row chunks (one unless M > kSkinnyMaxM, and then batch == 1): rows r0 .. r0 + rows - 1 of A's panel and of C
  for (int64_t r0 = 0; r0 < M; r0 += kSkinnyMaxM) {
    const int64_t rows = M - r0 < kSkinnyMaxM ? M - r0 : kSkinnyMaxM;
    const int64_t Mp = 32 * skinny_row_tiles(rows), cols = skinny_cols((int)(Mp / 32));
    int bps;
    const int slices = skinny_outer_slices((N + cols - 1) / cols * batch, K / kSkinnyBlockK, Mp, forced_slices, bps);
    const uint16_t* Ac = Ap + r0 * K;  // panel row blocks are contiguous: 32 rows x K values each
    float* Cc = C + r0 * ldc;
    auto go = [&]<int SK, bool ASYM>() {
      auto run = [&]<int MT>() {
        return launch_skinny<SK, ASYM, MT>(Ac, B_codes, B_scales, Cc, partial, rows, N, K, ldc, batch, slices, bps, s);
      };
      switch ((int)(Mp / 32)) {
        case 1: return run.template operator()<1>();
        case 2: return run.template operator()<2>();
        case 3: return run.template operator()<3>();
        case 4: return run.template operator()<4>();
        case 6: return run.template operator()<6>();
        default: return run.template operator()<8>();
      }
    };
    if (sk == kScaleE5M2)
      e = asym ? go.template operator()<kScaleE5M2, true>() : go.template operator()<kScaleE5M2, false>();
    else if (sk == kScaleE4M3)
      e = asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>();
    else
      e = asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
    if (e != hipSuccess) return e;
  }
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

}  // namespace amx
