// Fully quantized GEMM for ASYMMETRIC power-of-two scales (Eq. 1 with E8M0 scales, Sec. 4.2 "PoT") on the block-scaled
// matrix instruction with FP6 (E3M2) operands, which runs at the FP4 rate: one MFMA per 32x32x64 block, half the time
// of the FP8 form (gemm_fp8m.hip) and a quarter of the MFMAs of the sign-split FP4 form (gemm_fp4.hip).
//
// Merging. A group carries two power-of-two scales 2^sp, 2^sn (positive / negative elements). An E2M1 element is
// (1 or 1.5) * 2^k with k in -1 .. 2, and E3M2 holds (1 or 1.5) * 2^k exactly for k in -3 .. 4 (and 2^-4), so a group
// whose two scale exponents differ by at most 5 fits one FP6 operand exactly: with the larger exponent `top`, the
// class of the larger scale is moved up by u = max(0, diff - 3) <= 2 binades and the other one down by diff - u <= 3,
// and the block scale of the instruction is 2^(top - u). A class whose scale byte is 0 (2^-127: what the cast writes
// for a class without elements) is dropped; its elements are below 2^-124 in any case.
//
// Groups outside the window. Where some row's scales lie further apart, no common exponent serves both classes. Such a
// group position (the same K range in every row of the operand: outliers sit in channels, Sec. 3.1) is written
// TWICE along K, once with only its positive elements and their scale and once with only the negative ones - each is
// an MXFP4-like block, exact in FP6 - and the other operand repeats its group for the two copies; where both operands
// need it, A writes (a+, a+, a-, a-) and B (b+, b-, b+, b-). The sum over the lengthened K is the sum of Sec. 4.3
// term by term, so the GEMM kernel itself has one code path: a plain FP6 x FP6 product over K' >= K. Three small
// passes prepare it: which group positions need splitting (an OR over the rows of either operand), where each group
// lands in K' (a prefix sum), and the merge itself. K' is only known on the device, so the workspace is sized for the
// worst case (every position split in both operands, 4 K) and the kernel reads its trip count from memory.
//
// Layout. For FP6 operands lane l of the instruction holds row l % 32 and the 32-block l / 32 of the K step of 64:
// 32 six-bit elements, element p in bits 6 p .. 6 p + 5 of six registers, and supplies that block's scale byte
// (probed on the machine: the FP4 arrangement, not the FP8 one). A fragment (32 rows x K 64) is stored as
// [64 lanes][16 bytes] followed by [64 lanes][8 bytes] = 1536 bytes, the two aligned LDS reads that fill an operand.
// Panels: [row block of 32][K step][1536 bytes], rows padded to 256, K steps to a multiple of 12 with zero blocks.
// Anchors: [row block][K step / 4][64 lanes] words, byte q of lane 32 h + r = block scale of (row r, 32-block h) in
// K step 4 w + q.
//
// Static weights. B's panel as described depends on A (a position that A splits repeats B's group), so it is rebuilt on
// every call. For weights that stay, the three passes run once on B alone: the panel then holds B's own blocks (one
// per position, two where some row of B needs the split) and a call merges only A; its plan pass writes, per 32-block
// of K', where in B's panel that block lies, the GEMM kernel's PREP variant fetches B's blocks through that table,
// and a small pass puts B's anchors into the call's K' order. Same blocks in the same order: the same bits.
#include "device_formats.h"
#include "gemm_common.h"
#include "kernels.h"

namespace amx {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kFp6FragBytes = 1536;   // 64 lanes x 24 bytes
constexpr int kFp6StepPad = 12;       // K steps per row block are a multiple of this (ring of 6 stages, 4 steps per anchor word)
constexpr int kFp6FlagRows = 256;     // rows one workgroup of the flag pass ORs together
constexpr int kFp6Window = 5;         // largest difference of the two scale exponents one FP6 operand holds

static int64_t fp6_max_steps(int64_t K) { return round_up(2 * (K >> 5), kFp6StepPad); }  // every group split in both operands
static int64_t fp6_panel_bytes(int64_t rows_p, int64_t K) { return (rows_p / 32) * fp6_max_steps(K) * kFp6FragBytes; }
static int64_t fp6_anchor_bytes(int64_t rows_p, int64_t K) { return (rows_p / 32) * (fp6_max_steps(K) / 4) * 256; }
static int64_t fp6_flag_bytes(int64_t rows, int64_t K) { return ((rows + kFp6FlagRows - 1) / kFp6FlagRows) * (K >> 5); }
// per batch entry: positions (G + 1 words), split flags (G bytes, padded to words), the K step count
static int64_t fp6_plan_bytes(int64_t K) { return round_up(((K >> 5) + 1) * 4 + (K >> 5) + 4, 256); }

// B alone (prepared weights): at most every position split, 2 blocks each = K / 32 steps
static int64_t fp6_prepared_steps(int64_t K) { return round_up(K >> 5, kFp6StepPad); }
static int64_t fp6_prepared_panel_bytes(int64_t Np, int64_t K) { return (Np / 32) * fp6_prepared_steps(K) * kFp6FragBytes; }
static int64_t fp6_prepared_anchor_bytes(int64_t Np, int64_t K) { return (Np / 32) * (fp6_prepared_steps(K) / 4) * 256; }
// the table of B blocks behind the plan of a call on prepared weights: one word per 32-block of the lengthened K
static int64_t fp6_table_offset(int64_t K) { return fp6_plan_bytes(K); }
// (the kernel reads the entries of up to 16 stages past the last one: zeros)
static int64_t fp6_table_bytes(int64_t K) { return round_up(2 * (fp6_max_steps(K) + 17) * 4, 256); }

size_t fp6m_prepared_bytes(int64_t N, int64_t K) {
  const int64_t Np = round_up(N, kPanelRows);
  return (size_t)(fp6_prepared_panel_bytes(Np, K) + fp6_prepared_anchor_bytes(Np, K) + fp6_plan_bytes(K) +
                  round_up(fp6_flag_bytes(N, K), 256));
}

size_t fp6m_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows);
  return (size_t)(fp6_panel_bytes(Mp, K) + fp6_anchor_bytes(Mp, K) + fp6_anchor_bytes(Np, K) +
                  round_up(fp6_flag_bytes(M, K), 256) + fp6_plan_bytes(K) + fp6_table_bytes(K));
}

size_t fp6m_path_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch) {
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows);
  return (size_t)(batch * (fp6_panel_bytes(Mp, K) + fp6_panel_bytes(Np, K) + fp6_anchor_bytes(Mp, K) +
                           fp6_anchor_bytes(Np, K) + round_up(fp6_flag_bytes(M, K) + fp6_flag_bytes(N, K), 256) +
                           fp6_plan_bytes(K)));
}

// Does this pair of scale bytes need the split form? (a class with byte 0 is dropped, see above)
__device__ __forceinline__ bool fp6_out_of_window(uint32_t sp, uint32_t sn) {
  const uint32_t diff = sp > sn ? sp - sn : sn - sp;
  return sp != 0 && sn != 0 && diff > (uint32_t)kFp6Window;
}

// ---- pass 1: which group positions hold, in some row, scales too far apart -------------------------------------------
// grid: (ceil(G / 64), chunks of kFp6FlagRows rows of A + the same of B, batch); block 256 = 64 group positions x 4
// row lanes: a wave reads 64 consecutive scale pairs of one row; the four row lanes are ORed through LDS.
// flags: [batch][chunk][G] bytes, A's chunks then B's.
__global__ __launch_bounds__(256) void fp6_flag_kernel(const uint8_t* __restrict__ As, const uint8_t* __restrict__ Bs,
                                                       int64_t M, int64_t N, int64_t G, int chunks_a, int chunks_b,
                                                       uint8_t* __restrict__ flags) {
  __shared__ uint32_t any_lane[4][64];
  const bool second = (int)blockIdx.y >= chunks_a;
  const int chunk = (int)blockIdx.y - (second ? chunks_a : 0);
  const int64_t b = blockIdx.z, R = second ? N : M;
  const uint16_t* src = reinterpret_cast<const uint16_t*>(second ? Bs : As) + b * R * G;
  const int64_t r0 = (int64_t)chunk * kFp6FlagRows, r1 = r0 + kFp6FlagRows < R ? r0 + kFp6FlagRows : R;
  const int gx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int64_t g = (int64_t)blockIdx.x * 64 + gx;
  uint32_t any = 0;
  if (g < G) {
#pragma unroll 8
    for (int64_t r = r0 + ry; r < r1; r += 4) {
      const uint32_t s = src[r * G + g];
      any |= fp6_out_of_window(s & 255u, s >> 8) ? 1u : 0u;
    }
  }
  any_lane[ry][gx] = any;
  __syncthreads();
  if (ry == 0 && g < G)
    flags[(b * (chunks_a + chunks_b) + blockIdx.y) * G + g] =
        (uint8_t)(any_lane[0][gx] | any_lane[1][gx] | any_lane[2][gx] | any_lane[3][gx]);
}

// ---- pass 2: where every group lands in the lengthened K ---------------------------------------------------------------
// grid: (1, 1, batch); block 256. plan (per batch entry): pos[G + 1] words (first 32-block of group g; pos[G] = total
// blocks), then G bytes of split flags (bit 0: A's position is split, bit 1: B's), then - word aligned - the number
// of K steps (total blocks / 2 rounded up to a multiple of kFp6StepPad).
// With a prepared B (prepared_plan: the plan B's own passes left, pos and split of B alone): B's flags come from that
// plan instead of the flag array (chunks_b = 0), and a table at table_offset names, for every 32-block e of the
// lengthened K, the block i of B's prepared panel that stands there (zero-padding blocks: block 0, against A's zeros),
// as the byte offset of its 16-byte part within a row block of the panel, (i / 2) * 1536 + (i % 2) * 512, with i % 2
// in bit 0 (its 8-byte part lies at (i / 2) * 1536 + 1024 + (i % 2) * 256).
__global__ __launch_bounds__(256) void fp6_plan_kernel(const uint8_t* __restrict__ flags, int64_t G, int chunks_a,
                                                       int chunks_b, int64_t plan_stride, int64_t steps_offset,
                                                       uint8_t* __restrict__ plan_base,
                                                       const uint8_t* __restrict__ prepared_plan, int64_t table_offset) {
  __shared__ uint32_t part[256];
  __shared__ uint32_t totals[2];  // blocks in use, blocks after padding to whole K steps
  const int64_t b = blockIdx.z;
  const uint8_t* fl = flags + b * (chunks_a + chunks_b) * G;
  uint8_t* plan = plan_base + b * plan_stride;
  uint32_t* pos = reinterpret_cast<uint32_t*>(plan);
  uint8_t* split = plan + (G + 1) * 4;
  uint32_t* steps = reinterpret_cast<uint32_t*>(plan + steps_offset);
  // OR over the row chunks, all threads side by side, into LDS: one byte per group position (bit 0: A, bit 1: B)
  __shared__ uint32_t gathered[(1 << 15) / 4];  // K <= 2^20: at most 2^15 group positions
  const int64_t words = (G + 3) / 4;
  for (int64_t w = threadIdx.x; w < words; w += 256) gathered[w] = 0;
  __syncthreads();
  const int64_t total = (int64_t)(chunks_a + chunks_b) * G;
  if ((G & 3) == 0) {  // four flags per load
    const uint32_t* fl4 = reinterpret_cast<const uint32_t*>(fl);
    for (int64_t idx0 = threadIdx.x; idx0 < total / 4; idx0 += 8 * 256) {  // eight loads in flight per thread
      uint32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = idx0 + u * 256 < total / 4 ? fl4[idx0 + u * 256] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int64_t idx = idx0 + u * 256;
        if (v[u]) atomicOr(&gathered[idx % words], idx / words < chunks_a ? v[u] : v[u] << 1);
      }
    }
  } else {
    for (int64_t idx = threadIdx.x; idx < total; idx += 256)
      if (fl[idx]) atomicOr(&gathered[(idx % G) >> 2], (idx / G < chunks_a ? 1u : 2u) << (8 * (idx % G & 3)));
  }
  __syncthreads();
  if (prepared_plan) {  // B's flags: bit 1 of its own plan's split bytes
    const uint8_t* split_b = prepared_plan + (G + 1) * 4;
    for (int64_t g = threadIdx.x; g < G; g += 256)
      if (split_b[g] & 2u) atomicOr(&gathered[g >> 2], 2u << (8 * (g & 3)));
    __syncthreads();
  }
  auto flags_of = [&](int64_t g) { return (gathered[g >> 2] >> (8 * (g & 3))) & 3u; };
  for (int64_t g = threadIdx.x; g < G; g += 256) split[g] = (uint8_t)flags_of(g);
  const int64_t per = (G + 255) / 256, g0 = threadIdx.x * per, g1 = g0 + per < G ? g0 + per : G;
  uint32_t sum = 0;
  for (int64_t g = g0; g < g1; ++g) sum += (1u + (flags_of(g) & 1u)) * (1u + (flags_of(g) >> 1));
  // exclusive scan of the 256 partial sums: within each wave by lane shifts, then the four waves' totals (a serial
  // scan by one thread is a chain of 256 dependent LDS accesses, 9 of this pass's 10 microseconds)
  uint32_t incl = sum;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, 64);
    if ((int)(threadIdx.x & 63) >= d) incl += up;
  }
  if ((threadIdx.x & 63) == 63) part[threadIdx.x >> 6] = incl;  // the wave's total
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w < (int)(threadIdx.x >> 6)) before += part[w];
    all += part[w];
  }
  if (threadIdx.x == 0) {
    pos[G] = all;
    const uint32_t ks = (all + 1) / 2;
    steps[0] = (ks + kFp6StepPad - 1) / kFp6StepPad * kFp6StepPad;
    totals[0] = all, totals[1] = 2 * steps[0];
  }
  __syncthreads();
  uint32_t run = before + incl - sum;
  const uint32_t* pos_b = reinterpret_cast<const uint32_t*>(prepared_plan);
  uint32_t* table = reinterpret_cast<uint32_t*>(plan + table_offset);
  for (int64_t g = g0; g < g1; ++g) {
    pos[g] = run;
    const uint32_t fa = flags_of(g) & 1u, fb = flags_of(g) >> 1;
    if (prepared_plan) {  // A holds each sign class for as many blocks as B alternates: (b+, b-, b+, b-)
      const uint32_t b0 = pos_b[g];
      for (uint32_t e = 0; e < (1u + fa) * (1u + fb); ++e) {
        const uint32_t i = b0 + (fb ? (e & 1u) : 0u);  // block i of B's panel: step i / 2, lanes 32 (i % 2) ..
        table[run + e] = (i >> 1) * (uint32_t)kFp6FragBytes + (i & 1u) * 512u + (i & 1u);
      }
    }
    run += (1u + fa) * (1u + fb);
  }
  if (prepared_plan)  // the zero blocks that pad K, and the 17 stages the kernel's table reads may run past the end
    for (uint32_t e = totals[0] + threadIdx.x; e < totals[1] + 34; e += 256) table[e] = 0;
}

// ---- pass 3: the merge ---------------------------------------------------------------------------------------------------
// E3M2 patterns of the E2M1 magnitudes 0, .5, 1, 1.5 (low word) and 2, 3, 4, 6 (high word) moved by `shift` binades
// (-3 .. 2), one per byte. At shift 0 they are 00 08 0C 0E | 10 12 14 16; a binade is 4 in the pattern while the
// exponent field stays >= 1, and the few values below that are E3M2 subnormals (quarters of 2^-2): .5 * 2^-2 -> 02,
// and .5, 1, 1.5 at 2^-3 -> 01 02 03.
__device__ __forceinline__ void fp6_lut(int shift, uint32_t& lo, uint32_t& hi) {
  lo = shift >= -1 ? 0x0E0C0800u + (uint32_t)(shift * 0x04040400) : (shift == -2 ? 0x06040200u : 0x03020100u);
  hi = shift >= -2 ? 0x16141210u + (uint32_t)(shift * 0x04040404) : 0x0A080604u;
}

// The 32 codes of a group (four words of eight nibbles) -> six words of 32 six-bit elements (element p in bits
// 6 p .. 6 p + 5), through the two classes' pattern tables: a byte permute looks up four elements at a time.
__device__ __forceinline__ void fp6_convert(const uint32_t (&codes)[4], uint32_t pos_lo, uint32_t pos_hi, uint32_t neg_lo,
                                            uint32_t neg_hi, uint32_t (&w)[6]) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    uint32_t t[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t x = (codes[2 * half + (q >> 1)] >> (16 * (q & 1))) & 0xFFFFu;  // four nibbles ...
      x = (x | (x << 8)) & 0x00FF00FFu;
      x = (x | (x << 4)) & 0x0F0F0F0Fu;                                       // ... one per byte
      const uint32_t sel = x & 0x07070707u;
      const uint32_t pp = __builtin_amdgcn_perm(pos_hi, pos_lo, sel), pn = __builtin_amdgcn_perm(neg_hi, neg_lo, sel);
      const uint32_t is_neg = ((x >> 3) & 0x01010101u) * 0xFFu;
      const uint32_t y = (pn & is_neg) | (pp & ~is_neg);
      t[q] = (y & 0x3Fu) | ((y >> 2) & 0xFC0u) | ((y >> 4) & 0x3F000u) | ((y >> 6) & 0xFC0000u);  // 4 x 6 bits
    }
    w[3 * half] = t[0] | (t[1] << 24);
    w[3 * half + 1] = (t[1] >> 8) | (t[2] << 16);
    w[3 * half + 2] = (t[2] >> 16) | (t[3] << 8);
  }
}

// One merged 32-block of one row into the panel: block p of the lengthened K, fragment lane 32 * (p % 2) + row % 32.
__device__ __forceinline__ void fp6_store_block(const uint32_t (&w)[6], uint32_t anchor, uint8_t* frag_base,
                                                uint8_t* anchor_base, uint32_t p, int row_in_block) {
  const uint32_t step = p >> 1, lane = (p & 1u) * 32u + (uint32_t)row_in_block;
  uint8_t* f = frag_base + (int64_t)step * kFp6FragBytes;
  *reinterpret_cast<uint4*>(f + lane * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  *reinterpret_cast<uint2*>(f + 1024 + lane * 8) = make_uint2(w[4], w[5]);
  anchor_base[((int64_t)(step >> 2) * 64 + lane) * 4 + (step & 3u)] = (uint8_t)anchor;
}

// grid: (Rp / 32 of A + Rp / 32 of B, ceil((G + 2 kFp6StepPad) / 8), batch); block 256 = 32 rows x 8 group positions:
// wave w takes rows 8 w .. 8 w + 7, lane = 8 * (row % 8) + group, so that a wave reads eight whole 128-byte lines of
// codes and writes 128 contiguous bytes per fragment half. Group slots >= G write the zero blocks that pad K' to whole
// K steps.
struct Fp6MergeJob {
  const uint8_t* codes;
  const uint8_t* scales;
  uint8_t* panel;
  uint8_t* anchors;
  int64_t R, Rp;
};
__global__ __launch_bounds__(256) void fp6_merge_kernel(Fp6MergeJob ja, Fp6MergeJob jb, int64_t K, int64_t max_steps,
                                                        int64_t plan_stride, int64_t steps_offset,
                                                        const uint8_t* __restrict__ plan_base) {
  const int64_t G = K >> 5, b = blockIdx.z;
  const bool second = (int64_t)blockIdx.x >= ja.Rp / 32;
  const Fp6MergeJob& job = second ? jb : ja;
  const int64_t rb = (int64_t)blockIdx.x - (second ? ja.Rp / 32 : 0);
  const int row_in_block = 8 * (threadIdx.x >> 6) + ((threadIdx.x & 63) >> 3);
  const int64_t r = rb * 32 + row_in_block, g = (int64_t)blockIdx.y * 8 + (threadIdx.x & 7);
  const uint8_t* plan = plan_base + b * plan_stride;
  const uint32_t* pos = reinterpret_cast<const uint32_t*>(plan);
  const uint8_t* split = plan + (G + 1) * 4;
  const uint32_t steps = *reinterpret_cast<const uint32_t*>(plan + steps_offset);
  uint8_t* frag_base = job.panel + (b * (job.Rp / 32) + rb) * max_steps * kFp6FragBytes;
  uint8_t* anchor_base = job.anchors + (b * (job.Rp / 32) + rb) * (max_steps / 4) * 256;
  uint32_t w[6] = {0, 0, 0, 0, 0, 0};
  if (g >= G) {  // padding blocks behind the last group
    const uint32_t p = pos[G] + (uint32_t)(g - G);
    if (p < 2 * steps) fp6_store_block(w, 0, frag_base, anchor_base, p, row_in_block);
    return;
  }
  uint32_t codes[4] = {0, 0, 0, 0};
  uint32_t sp = 0, sn = 0;
  if (r < job.R) {
    const uint4 c = *reinterpret_cast<const uint4*>(job.codes + (b * job.R + r) * (K >> 1) + g * 16);
    codes[0] = c.x, codes[1] = c.y, codes[2] = c.z, codes[3] = c.w;
    const uint32_t sb = *reinterpret_cast<const uint16_t*>(job.scales + ((b * job.R + r) * G + g) * 2);
    sp = sb & 255u, sn = sb >> 8;
  }
  const uint32_t p = pos[g], sf = split[g];
  const bool mine = second ? (sf & 2u) != 0 : (sf & 1u) != 0, other = second ? (sf & 1u) != 0 : (sf & 2u) != 0;
  uint32_t pos_lo, pos_hi, neg_lo, neg_hi;
  if (!mine) {
    // both classes in one block; a dropped class (scale byte 0) takes the other's exponent and is written as zeros
    const uint32_t ep = sp ? sp : sn, en = sn ? sn : sp;
    const uint32_t top = ep > en ? ep : en, diff = ep > en ? ep - en : en - ep;  // <= kFp6Window here
    const uint32_t up = diff > 3u ? diff - 3u : 0u, anchor = top - up;
    fp6_lut((int)ep - (int)anchor, pos_lo, pos_hi);
    fp6_lut((int)en - (int)anchor, neg_lo, neg_hi);
    if (sp == 0 && sn != 0) pos_lo = pos_hi = 0;
    if (sn == 0 && sp != 0) neg_lo = neg_hi = 0;
    fp6_convert(codes, pos_lo, pos_hi, neg_lo | 0x20202020u, neg_hi | 0x20202020u, w);
    fp6_store_block(w, anchor, frag_base, anchor_base, p, row_in_block);
    if (other) fp6_store_block(w, anchor, frag_base, anchor_base, p + 1, row_in_block);
    return;
  }
  // split position: positive elements with their scale, negative elements with theirs. The first operand holds each
  // sign class for as many blocks as the second one alternates: A (a+, a+, a-, a-), B (b+, b-, b+, b-).
  uint32_t wn[6];
  fp6_lut(0, pos_lo, pos_hi);
  fp6_convert(codes, pos_lo, pos_hi, 0u, 0u, w);                                    // the positive elements alone
  fp6_convert(codes, 0u, 0u, pos_lo | 0x20202020u, pos_hi | 0x20202020u, wn);      // the negative elements alone
  if (!other) {
    fp6_store_block(w, sp, frag_base, anchor_base, p, row_in_block);
    fp6_store_block(wn, sn, frag_base, anchor_base, p + 1, row_in_block);
  } else if (!second) {
    fp6_store_block(w, sp, frag_base, anchor_base, p, row_in_block);
    fp6_store_block(w, sp, frag_base, anchor_base, p + 1, row_in_block);
    fp6_store_block(wn, sn, frag_base, anchor_base, p + 2, row_in_block);
    fp6_store_block(wn, sn, frag_base, anchor_base, p + 3, row_in_block);
  } else {
    fp6_store_block(w, sp, frag_base, anchor_base, p, row_in_block);
    fp6_store_block(wn, sn, frag_base, anchor_base, p + 1, row_in_block);
    fp6_store_block(w, sp, frag_base, anchor_base, p + 2, row_in_block);
    fp6_store_block(wn, sn, frag_base, anchor_base, p + 3, row_in_block);
  }
}

// Prepared B: its anchors in the order of this call's lengthened K. grid: (Np / 32, ceil(words / 4)); block 256 = four
// anchor words x 64 lanes. Word w of lane 32 h + r holds, in byte q, the block scale of (row r, 32-block h) of K step
// 4 w + q, i.e. of block e = 2 (4 w + q) + h, which is block table[e] of the prepared panel; steps beyond the call's
// count get byte 0 (they multiply A's zero blocks).
__global__ __launch_bounds__(256) void fp6_gather_anchors_kernel(const uint8_t* __restrict__ prepared_anchors,
                                                                 int64_t prepared_words, const uint8_t* __restrict__ plan,
                                                                 int64_t steps_offset, int64_t table_offset,
                                                                 int64_t max_words, uint8_t* __restrict__ out) {
  const uint32_t steps = *reinterpret_cast<const uint32_t*>(plan + steps_offset);
  const uint32_t* table = reinterpret_cast<const uint32_t*>(plan + table_offset);
  const int64_t rb = blockIdx.x, w = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
  const uint32_t slot = threadIdx.x & 63, h = slot >> 5, r = slot & 31;
  if (w >= max_words) return;
  const uint8_t* src = prepared_anchors + rb * prepared_words * 256;
  uint32_t word = 0;
#pragma unroll
  for (uint32_t q = 0; q < 4; ++q) {
    const uint32_t step = (uint32_t)w * 4 + q;
    if (step < steps) {
      const uint32_t t = table[2 * step + h], odd = t & 1u, istep = t / (uint32_t)kFp6FragBytes;
      word |= (uint32_t)src[((int64_t)(istep >> 2) * 64 + odd * 32 + r) * 4 + (istep & 3u)] << (8 * q);
    }
  }
  reinterpret_cast<uint32_t*>(out)[(rb * max_words + w) * 64 + slot] = word;
}

// ---- the GEMM ------------------------------------------------------------------------------------------------------------
// 256 x 256 tile, 2 x 2 waves of 4 x 4 MFMA tiles. One stage = one K step of 64: 16 fragments = 24 KiB; six stage
// arrays form the ring: while stage S is multiplied, stage S + 1 is complete in LDS (fragment reads run ahead into it)
// and stages S + 2 .. S + 5 are in flight as direct-to-LDS loads (the panels are fragment-major, so staging is a linear
// copy of 1 KiB pieces). One barrier per stage.
// GLU: the gated-activation epilogue of store_glu_tiles() (gemm_common.h); C is then the BF16 output [M][ldc].
// PREP: B comes from a prepared panel (B's own blocks, independent of A): b_steps K steps per row block, and the plan
// holds, behind the step count, the table of B blocks of the lengthened K; Bsc is this call's gathered anchor array.
template <int WM, int WN, int FM, int FN, bool GLU = false, bool PREP = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_fp6m_kernel(const uint8_t* __restrict__ Ap,
                                                                 const uint8_t* __restrict__ Asc,
                                                                 const uint8_t* __restrict__ Bp,
                                                                 const uint8_t* __restrict__ Bsc,
                                                                 const uint8_t* __restrict__ plan_base,
                                                                 int64_t plan_stride, int64_t plan_steps_offset,
                                                                 float* __restrict__ C, int64_t M, int64_t N, int64_t Mp,
                                                                 int64_t Np, int max_steps, int64_t ldc, int tiles_m,
                                                                 int tiles_n, int super_m, int b_steps,
                                                                 int64_t plan_table_offset) {
  static_assert(WM == 2 && WN == 2 && FM == 4 && FN == 4, "the issue schedule is written for 2 x 2 waves of 4 x 4 tiles");
  constexpr int kWaves = WM * WN, kRowBlocks = 8;           // row blocks of 32 per operand and tile
  constexpr int kStageBytes = 2 * kRowBlocks * kFp6FragBytes;  // 24 KiB
  constexpr int kLoads = kStageBytes / 1024 / kWaves;          // 6 direct-to-LDS loads per wave and stage
  __shared__ __attribute__((aligned(1024))) uint8_t lds0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds1[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds2[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds3[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds4[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t lds5[kStageBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int64_t b = blockIdx.z;
  int tm, tn;
  if (!tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, super_m, tm, tn)) return;  // uniform, before any barrier

  // the K steps of this batch entry (a multiple of 12, written by the plan pass)
  // (clamped to the panel's capacity, so that no value found there can run the loop past it)
  const uint32_t planned = *reinterpret_cast<const uint32_t*>(plan_base + b * plan_stride + plan_steps_offset);
  const int nsteps = __builtin_amdgcn_readfirstlane((int)(planned < (uint32_t)max_steps ? planned : (uint32_t)max_steps));
  const int nwords = nsteps >> 2;
  const int64_t step_bytes = kFp6FragBytes;
  const uint8_t* Abase = Ap + ((b * (Mp >> 5) + (int64_t)tm * kRowBlocks) * max_steps) * step_bytes;
  const int b_panel_steps = PREP ? b_steps : max_steps;  // K steps a row block of B's panel holds
  const uint8_t* Bbase = Bp + ((b * (Np >> 5) + (int64_t)tn * kRowBlocks) * b_panel_steps) * step_bytes;
  const uint32_t panel_span = (uint32_t)kRowBlocks * (uint32_t)max_steps * (uint32_t)kFp6FragBytes;
  const uint32_t b_span = (uint32_t)kRowBlocks * (uint32_t)b_panel_steps * (uint32_t)kFp6FragBytes;
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(Abase), 0, (int)panel_span, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(Bbase), 0, (int)b_span, 0x00020000);
  const int max_words = max_steps >> 2;
  const __amdgpu_buffer_rsrc_t Asr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Asc + ((b * (Mp >> 5) + (int64_t)tm * kRowBlocks + wm * FM) * max_words) * 256), 0,
      FM * max_words * 256, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bsc + ((b * (Np >> 5) + (int64_t)tn * kRowBlocks + wn * FN) * max_words) * 256), 0,
      FN * max_words * 256, 0x00020000);

  // Load L (0 .. 5) of this wave copies KiB f = wave + 4 L of a stage: f < 12 lies in A's eight fragments, the rest in
  // B's. A KiB straddles fragments (1536 bytes each), so the source offset is per lane: byte x of the operand's half
  // stage belongs to row block x / 1536, whose K steps lie max_steps fragments apart in the panel.
  // (wave + 4 L) % 12 takes three values, wave, wave + 4 and wave + 8, the same for A's loads (L < 3) and B's. Named
  // variables, not an array: an array element among the builtin's arguments trips the host pass of the compiler,
  // which then drops the kernel's launch stub.
  auto source_offset = [&](int chunk) {
    const int x = chunk * 1024 + lane * 16;
    return (x / kFp6FragBytes) * max_steps * kFp6FragBytes + x % kFp6FragBytes;
  };
  const int src0 = source_offset(wave), src1 = source_offset(wave + kWaves), src2 = source_offset(wave + 2 * kWaves);
#define AMX_SRC(L) ((L) % 3 == 0 ? src0 : (L) % 3 == 1 ? src1 : src2)
  // PREP: the two 32-blocks of a stage come from anywhere in B's panel, so B's half stage is laid out differently in
  // LDS: the eight fragments' 16-byte parts first ([8][64 lanes][16 bytes]: lanes 0-31 the stage's first block, 32-63
  // its second), then their 8-byte parts ([8][64 lanes][8 bytes]). KiB 0 .. 7 of the half stage are then the 16-byte
  // parts of row blocks 0 .. 7, KiB 8 + j the 8-byte parts of row blocks 2 j (lanes 0-31 of the load: 16-byte pieces
  // 0-15 first block, 16-31 second) and 2 j + 1 (lanes 32-63). A wave's three loads are KiB wave, wave + 4 (16-byte
  // parts) and wave + 8 (8-byte parts). Per lane and load, loop-invariant: the source offset without the block (pb*)
  // and whether the lane takes the stage's second block (ps*); per stage, from the table: the two blocks' offsets.
  int pb0 = 0, pb1 = 0, pb2 = 0;
  bool ps0 = false, ps1 = false, ps2 = false;
  if constexpr (PREP) {
    const int row_block_bytes = b_panel_steps * kFp6FragBytes;
    pb0 = wave * row_block_bytes + (lane & 31) * 16, ps0 = lane >= 32;
    pb1 = (wave + kWaves) * row_block_bytes + (lane & 31) * 16, ps1 = lane >= 32;
    pb2 = (2 * wave + (lane >> 5)) * row_block_bytes + 1024 + (lane & 15) * 16, ps2 = (lane & 31) >= 16;
  }
  const uint32_t* table = reinterpret_cast<const uint32_t*>(plan_base + b * plan_stride + plan_table_offset);
#define AMX_PB(L) ((L) % 3 == 0 ? pb0 : (L) % 3 == 1 ? pb1 : pb2)
#define AMX_PS(L) ((L) % 3 == 0 ? ps0 : (L) % 3 == 1 ? ps1 : ps2)
  // T0, T1: the table entries of stage ST's two blocks (PREP only): offset of the 16-byte part, parity in bit 0; the
  // 8-byte part of an odd block lies 256 bytes, not 512, behind the even one's
#define AMX_PART(L, T) ((L) % 3 == 2 ? ((T) & ~1u) - ((T) & 1u) * 256u : ((T) & ~1u))
#define AMX_ISSUE_LOAD(L, ST, DST, T0, T1)                                                                  \
  {                                                                                                         \
    if ((L) < kLoads / 2) {                                                                                 \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + (wave + kWaves * (L)) * 1024), 16,   \
                                               AMX_SRC(L), (ST) * kFp6FragBytes, 0, 0);                     \
    } else if constexpr (PREP) {                                                                            \
      const int voff_ = AMX_PB(L) + (int)(AMX_PS(L) ? AMX_PART(L, T1) : AMX_PART(L, T0));                   \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)((DST) + (wave + kWaves * (L)) * 1024), 16,   \
                                               voff_, 0, 0, 0);                                             \
    } else {                                                                                                \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)((DST) + (wave + kWaves * (L)) * 1024), 16,   \
                                               AMX_SRC(L), (ST) * kFp6FragBytes, 0, 0);                     \
    }                                                                                                       \
  }
  // anchor words of four K steps (word W) into register set SET (three sets: the loop body covers three words)
  uint32_t sa[3][FM], sb[3][FN];
#define AMX_LOAD_ANCHORS(SET, W)                                                                        \
  {                                                                                                     \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) sa[SET][i] =                                         \
        __builtin_amdgcn_raw_buffer_load_b32(Asr, lane * 4, (i * max_words + (W)) * 256, 0);            \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) sb[SET][j] =                                         \
        __builtin_amdgcn_raw_buffer_load_b32(Bsr, lane * 4, (j * max_words + (W)) * 256, 0);            \
  }

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // prologue: the anchors of the first word, then five stages in flight; stages 0 and 1 must have landed
  AMX_LOAD_ANCHORS(0, 0);
  uint32_t tp[12];  // table entries of stages 0 .. 5 (nsteps >= 12)
#pragma unroll
  for (int e = 0; e < 12; ++e) tp[e] = PREP ? table[e] : 0u;
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 0, lds0, tp[0], tp[1]);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 1, lds1, tp[2], tp[3]);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 2, lds2, tp[4], tp[5]);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 3, lds3, tp[6], tp[7]);
#pragma unroll
  for (int l = 0; l < kLoads; ++l) AMX_ISSUE_LOAD(l, 4, lds4, tp[8], tp[9]);

  AMX_WAIT_VMCNT(3 * kLoads);
  AMX_BARRIER();

  // operand registers: a fragment is 16 + 8 bytes per lane. A of step i in aR[i & 1] (read one step ahead), B of stage
  // S in bR[S & 1] (read during stage S - 1)
  struct Frag {
    u32x4 lo;
    u32x2 hi;
  };
  Frag aR[2], bR[2][FN];
  const int offA = (wm * FM) * kFp6FragBytes, offB = (kRowBlocks + wn * FN) * kFp6FragBytes;
  // B fragment j of this wave: 16-byte parts at b_lo + j * b_lo_step, 8-byte parts at b_hi + j * b_hi_step (stage base
  // and lane offsets included below)
  constexpr int kHalf = kRowBlocks * kFp6FragBytes;
  const int b_lo = PREP ? kHalf + wn * FN * 1024 : offB, b_hi = PREP ? kHalf + kRowBlocks * 1024 + wn * FN * 512 - 1024 : offB;
  constexpr int b_lo_step = PREP ? 1024 : kFp6FragBytes, b_hi_step = PREP ? 512 : kFp6FragBytes;
  const int lo_off = lane * 16, hi_off = 1024 + lane * 8;
#define AMX_RD_LO(P) (*reinterpret_cast<const u32x4*>(P))
#define AMX_RD_HI(P) (*reinterpret_cast<const u32x2*>(P))
#define AMX_OPERAND(F) \
  i32x8 { (int)(F).lo.x, (int)(F).lo.y, (int)(F).lo.z, (int)(F).lo.w, (int)(F).hi.x, (int)(F).hi.y, 0, 0 }
  aR[0].lo = AMX_RD_LO(lds0 + offA + lo_off);
  aR[0].hi = AMX_RD_HI(lds0 + offA + hi_off);
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    bR[0][j].lo = AMX_RD_LO(lds0 + b_lo + j * b_lo_step + lo_off);
    bR[0][j].hi = AMX_RD_HI(lds0 + b_hi + j * b_hi_step + hi_off);
  }

  // Stage S = K step Q (0..3, a literal: it selects the anchor byte) of the word in set SET; B operands in set BSET;
  // CUR / NXT: the arrays of stage S and S + 1; FETCH: the array stage S + 5 lands in (read last during stage S - 1).
  // Step i (A row block i): slot 0 reads the A fragment of step i + 1 (of the next stage's step 0 when i = 3), slot 1
  // the B fragment i of the next stage, slots 2 and 3 issue this step's share of the direct-to-LDS loads; the first
  // stage of a word also requests the next word's anchors (set NSET, word clamped at the end).
#define AMX_STAGE(S, SET, NSET, Q, BSET, CUR, NXT, FETCH)                                                        \
  {                                                                                                              \
    const int fetch_ = (S) + 5 < nsteps ? (S) + 5 : nsteps - 1;                                                  \
    if constexpr ((Q) == 0) {                                                                                    \
      const int w_ = ((S) >> 2) + 1 < nwords ? ((S) >> 2) + 1 : nwords - 1;                                      \
      AMX_LOAD_ANCHORS(NSET, w_);                                                                                \
    }                                                                                                            \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                                             \
      const i32x8 av = AMX_OPERAND(aR[i & 1]);                                                                   \
      {                                                                                                          \
        const uint8_t* src_ = i + 1 < FM ? (CUR) : (NXT);                                                        \
        const int i2 = (i + 1) % FM;                                                                             \
        aR[(i + 1) & 1].lo = AMX_RD_LO(src_ + offA + i2 * kFp6FragBytes + lo_off);                               \
        aR[(i + 1) & 1].hi = AMX_RD_HI(src_ + offA + i2 * kFp6FragBytes + hi_off);                               \
      }                                                                                                          \
      acc[i][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, AMX_OPERAND(bR[BSET][0]), acc[i][0], 3, 3, \
                                                                  Q, (int)sa[SET][i], Q, (int)sb[SET][0]);       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      bR[(BSET) ^ 1][i].lo = AMX_RD_LO((NXT) + b_lo + i * b_lo_step + lo_off);                                   \
      bR[(BSET) ^ 1][i].hi = AMX_RD_HI((NXT) + b_hi + i * b_hi_step + hi_off);                                   \
      acc[i][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, AMX_OPERAND(bR[BSET][1]), acc[i][1], 3, 3, \
                                                                  Q, (int)sa[SET][i], Q, (int)sb[SET][1]);       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      AMX_ISSUE_LOAD(i, fetch_, FETCH, tt[2 * ((S) - s)], tt[2 * ((S) - s) + 1]);                                \
      acc[i][2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, AMX_OPERAND(bR[BSET][2]), acc[i][2], 3, 3, \
                                                                  Q, (int)sa[SET][i], Q, (int)sb[SET][2]);       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      if (i + FM < kLoads) AMX_ISSUE_LOAD(i + FM, fetch_, FETCH, tt[2 * ((S) - s)], tt[2 * ((S) - s) + 1]);      \
      acc[i][3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, AMX_OPERAND(bR[BSET][3]), acc[i][3], 3, 3, \
                                                                  Q, (int)sa[SET][i], Q, (int)sb[SET][3]);       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    /* stage S + 2 must be complete before stage S + 1 reads ahead into it: everything but the loads of the last   \
       three stages, and the anchor loads that were issued among them (in this stage or the one before) */         \
    AMX_WAIT_VMCNT(3 * kLoads + ((Q) < 2 ? FM + FN : 0));                                                        \
    AMX_BARRIER();                                                                                               \
  }

  for (int s = 0; s < nsteps; s += 12) {
    // PREP: the table entries of the twelve stages this round fetches (stages s + 5 .. s + 16), read as scalars in one
    // go: a scalar load's result is waited for together with every LDS read in flight, once per round instead of once
    // per stage. Stages past the end read the zeros behind the table's last entry (block 0, into a buffer that is
    // never multiplied).
    uint32_t tt[24];
#pragma unroll
    for (int e = 0; e < 24; ++e) tt[e] = PREP ? table[2 * (s + 5) + e] : 0u;
    AMX_STAGE(s, 0, 1, 0, 0, lds0, lds1, lds5);
    AMX_STAGE(s + 1, 0, 1, 1, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 2, 0, 1, 2, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 3, 0, 1, 3, 1, lds3, lds4, lds2);
    AMX_STAGE(s + 4, 1, 2, 0, 0, lds4, lds5, lds3);
    AMX_STAGE(s + 5, 1, 2, 1, 1, lds5, lds0, lds4);
    AMX_STAGE(s + 6, 1, 2, 2, 0, lds0, lds1, lds5);
    AMX_STAGE(s + 7, 1, 2, 3, 1, lds1, lds2, lds0);
    AMX_STAGE(s + 8, 2, 0, 0, 0, lds2, lds3, lds1);
    AMX_STAGE(s + 9, 2, 0, 1, 1, lds3, lds4, lds2);
    AMX_STAGE(s + 10, 2, 0, 2, 0, lds4, lds5, lds3);
    AMX_STAGE(s + 11, 2, 0, 3, 1, lds5, lds0, lds4);
  }
  AMX_WAIT_VMCNT(0);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_OPERAND
#undef AMX_RD_LO
#undef AMX_RD_HI
#undef AMX_LOAD_ANCHORS
#undef AMX_ISSUE_LOAD
#undef AMX_PB
#undef AMX_PS
#undef AMX_PART
#undef AMX_SRC

  if constexpr (GLU) {
    // every wave is past its last fragment read: four of the operand stages become the waves' transposition space
    static_assert(kWaves <= 4 && glu_stage_bytes<FM, FN>() <= kStageBytes, "stage too small");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    AMX_BARRIER();
    const int w = wm * WN + wn;
    uint8_t* stage = w == 0 ? lds0 : w == 1 ? lds1 : w == 2 ? lds2 : lds3;
    store_glu_tiles<FM, FN>(acc, stage, reinterpret_cast<uint16_t*>(C) + b * M * ldc, M, N >> 1, ldc,
                            (int64_t)tm * (32 * FM * WM) + wm * FM * 32, (int64_t)tn * (32 * FN * WN) + wn * FN * 32);
  } else
    store_c_tiles<FM, FN>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * (32 * FM * WM) + wm * FM * 32,
                          (int64_t)tn * (32 * FN * WN) + wn * FN * 32);
}

bool fp6m_path_supported(int64_t M, int64_t N, int64_t K) {
  // 32-bit byte offsets inside a tile's eight row blocks of the worst-case panel
  return M > 0 && N > 0 && K >= 32 && 8 * fp6_max_steps(K) * kFp6FragBytes < (int64_t(1) << 31);
}

hipError_t launch_gemm_fp6m_path(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                 const uint8_t* B_codes, const uint8_t* B_scales, float* C, int64_t ldc, int64_t batch,
                                 void* workspace, hipStream_t s, const KernelTimer& timer, bool glu) {
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows), G = K >> 5;
  const int64_t max_steps = fp6_max_steps(K);
  uint8_t* Ap = reinterpret_cast<uint8_t*>(workspace);
  uint8_t* Bp = Ap + batch * fp6_panel_bytes(Mp, K);
  uint8_t* Asc = Bp + batch * fp6_panel_bytes(Np, K);
  uint8_t* Bsc = Asc + batch * fp6_anchor_bytes(Mp, K);
  uint8_t* flags = Bsc + batch * fp6_anchor_bytes(Np, K);
  uint8_t* plan = flags + batch * round_up(fp6_flag_bytes(M, K) + fp6_flag_bytes(N, K), 256);
  const int chunks_a = (int)((M + kFp6FlagRows - 1) / kFp6FlagRows), chunks_b = (int)((N + kFp6FlagRows - 1) / kFp6FlagRows);
  const int64_t plan_stride = fp6_plan_bytes(K), steps_offset = round_up((G + 1) * 4 + G, 4);
  // (the flag array of one batch entry is (chunks_a + chunks_b) * G bytes; entries lie back to back)
  hipLaunchKernelGGL(fp6_flag_kernel, dim3((unsigned)((G + 63) / 64), (unsigned)(chunks_a + chunks_b), (unsigned)batch),
                     dim3(256), 0, s,
                     A_scales, B_scales, M, N, G, chunks_a, chunks_b, flags);
  hipLaunchKernelGGL(fp6_plan_kernel, dim3(1, 1, (unsigned)batch), dim3(256), 0, s, flags, G, chunks_a, chunks_b,
                     plan_stride, steps_offset, plan, static_cast<const uint8_t*>(nullptr), (int64_t)0);
  const Fp6MergeJob ja = {A_codes, A_scales, Ap, Asc, M, Mp}, jb = {B_codes, B_scales, Bp, Bsc, N, Np};
  hipLaunchKernelGGL(fp6_merge_kernel,
                     dim3((unsigned)((Mp + Np) / 32), (unsigned)((G + 2 * kFp6StepPad + 7) / 8), (unsigned)batch),
                     dim3(256), 0, s, ja, jb, K, max_steps, plan_stride, steps_offset, plan);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  using Cfg = TileCfg<2, 2, 4, 4>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  const int steps_cap = (int)max_steps;
  if (glu)
    hipLaunchKernelGGL((gemm_fp6m_kernel<2, 2, 4, 4, true>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s,
                       Ap, Asc, Bp, Bsc, plan, plan_stride, steps_offset, C, M, N, Mp, Np, steps_cap, ldc, tiles_m,
                       tiles_n, super_m, 0, (int64_t)0);
  else
    hipLaunchKernelGGL((gemm_fp6m_kernel<2, 2, 4, 4>), dim3(grid, 1, (unsigned)batch), dim3(Cfg::kThreads), 0, s, Ap,
                       Asc, Bp, Bsc, plan, plan_stride, steps_offset, C, M, N, Mp, Np, steps_cap, ldc, tiles_m, tiles_n,
                       super_m, 0, (int64_t)0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

// ---- prepared weights ------------------------------------------------------------------------------------------------
// prepared: [B's panel: its own blocks, one per position and two (b+, b-) where some row of B leaves the window]
// [its anchors][its plan: pos, split][scratch: its flag array]. The three passes above, run on B alone.
hipError_t launch_fp6m_prepare_b(int64_t N, int64_t K, const uint8_t* B_codes, const uint8_t* B_scales, void* prepared,
                                 hipStream_t s) {
  const int64_t Np = round_up(N, kPanelRows), G = K >> 5, b_steps = fp6_prepared_steps(K);
  uint8_t* Bp = reinterpret_cast<uint8_t*>(prepared);
  uint8_t* Bsc = Bp + fp6_prepared_panel_bytes(Np, K);
  uint8_t* plan = Bsc + fp6_prepared_anchor_bytes(Np, K);
  uint8_t* flags = plan + fp6_plan_bytes(K);
  const int chunks_b = (int)((N + kFp6FlagRows - 1) / kFp6FlagRows);
  const int64_t steps_offset = round_up((G + 1) * 4 + G, 4);
  hipLaunchKernelGGL(fp6_flag_kernel, dim3((unsigned)((G + 63) / 64), (unsigned)chunks_b, 1), dim3(256), 0, s,
                     static_cast<const uint8_t*>(nullptr), B_scales, (int64_t)0, N, G, 0, chunks_b, flags);
  hipLaunchKernelGGL(fp6_plan_kernel, dim3(1, 1, 1), dim3(256), 0, s, flags, G, 0, chunks_b, fp6_plan_bytes(K),
                     steps_offset, plan, static_cast<const uint8_t*>(nullptr), (int64_t)0);
  const Fp6MergeJob none = {nullptr, nullptr, nullptr, nullptr, 0, 0}, jb = {B_codes, B_scales, Bp, Bsc, N, Np};
  hipLaunchKernelGGL(fp6_merge_kernel, dim3((unsigned)(Np / 32), (unsigned)((G + 2 * kFp6StepPad + 7) / 8), 1), dim3(256), 0,
                     s, none, jb, K, b_steps, fp6_plan_bytes(K), steps_offset, plan);
  return hipGetLastError();
}

hipError_t launch_gemm_fp6m_prepared(int64_t M, int64_t N, int64_t K, const uint8_t* A_codes, const uint8_t* A_scales,
                                     const void* prepared, float* C, int64_t ldc, void* workspace, hipStream_t s,
                                     const KernelTimer& timer, bool glu) {
  const int64_t Mp = round_up(M, kPanelRows), Np = round_up(N, kPanelRows), G = K >> 5;
  const int64_t max_steps = fp6_max_steps(K), b_steps = fp6_prepared_steps(K);
  const uint8_t* Bp = reinterpret_cast<const uint8_t*>(prepared);
  const uint8_t* Bsc_prepared = Bp + fp6_prepared_panel_bytes(Np, K);
  const uint8_t* plan_b = Bsc_prepared + fp6_prepared_anchor_bytes(Np, K);
  uint8_t* Ap = reinterpret_cast<uint8_t*>(workspace);
  uint8_t* Asc = Ap + fp6_panel_bytes(Mp, K);
  uint8_t* Bsc = Asc + fp6_anchor_bytes(Mp, K);
  uint8_t* flags = Bsc + fp6_anchor_bytes(Np, K);
  uint8_t* plan = flags + round_up(fp6_flag_bytes(M, K), 256);
  const int chunks_a = (int)((M + kFp6FlagRows - 1) / kFp6FlagRows);
  const int64_t plan_stride = fp6_plan_bytes(K) + fp6_table_bytes(K), steps_offset = round_up((G + 1) * 4 + G, 4);
  const int64_t table_offset = fp6_table_offset(K);
  hipLaunchKernelGGL(fp6_flag_kernel, dim3((unsigned)((G + 63) / 64), (unsigned)chunks_a, 1), dim3(256), 0, s, A_scales,
                     static_cast<const uint8_t*>(nullptr), M, (int64_t)0, G, chunks_a, 0, flags);
  hipLaunchKernelGGL(fp6_plan_kernel, dim3(1, 1, 1), dim3(256), 0, s, flags, G, chunks_a, 0, plan_stride, steps_offset, plan,
                     plan_b, table_offset);
  const Fp6MergeJob ja = {A_codes, A_scales, Ap, Asc, M, Mp}, none = {nullptr, nullptr, nullptr, nullptr, 0, 0};
  hipLaunchKernelGGL(fp6_merge_kernel, dim3((unsigned)(Mp / 32), (unsigned)((G + 2 * kFp6StepPad + 7) / 8), 1), dim3(256), 0,
                     s, ja, none, K, max_steps, plan_stride, steps_offset, plan);
  const int64_t max_words = max_steps / 4;
  hipLaunchKernelGGL(fp6_gather_anchors_kernel, dim3((unsigned)(Np / 32), (unsigned)((max_words + 3) / 4)), dim3(256), 0, s,
                     Bsc_prepared, b_steps / 4, plan, steps_offset, table_offset, max_words, Bsc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  using Cfg = TileCfg<2, 2, 4, 4>;
  const int tiles_m = (int)((M + Cfg::kTileM - 1) / Cfg::kTileM), tiles_n = (int)((N + Cfg::kTileN - 1) / Cfg::kTileN);
  int super_m;
  const unsigned grid = supertile_grid(tiles_m, tiles_n, super_m);
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  const int steps_cap = (int)max_steps, b_cap = (int)b_steps;
  if (glu)
    hipLaunchKernelGGL((gemm_fp6m_kernel<2, 2, 4, 4, true, true>), dim3(grid, 1, 1), dim3(Cfg::kThreads), 0, s, Ap, Asc, Bp,
                       Bsc, plan, plan_stride, steps_offset, C, M, N, Mp, Np, steps_cap, ldc, tiles_m, tiles_n, super_m,
                       b_cap, table_offset);
  else
    hipLaunchKernelGGL((gemm_fp6m_kernel<2, 2, 4, 4, false, true>), dim3(grid, 1, 1), dim3(Cfg::kThreads), 0, s, Ap, Asc, Bp,
                       Bsc, plan, plan_stride, steps_offset, C, M, N, Mp, Np, steps_cap, ldc, tiles_m, tiles_n, super_m,
                       b_cap, table_offset);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

}  // namespace amx
