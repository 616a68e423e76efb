// Fused quantized attention for FEW queries against many keys (decoding: one or a handful of new tokens against a long
// key / value cache). Same per-tile arithmetic as attention.hip (Sec. 5.1 quantizes Q.K^T and the attention map times V;
// online softmax over key tiles of 32, each tile of probabilities cast as one group per query), but organised for the
// shape: the work is reading K and V once, so
//   - K and V are read as they are stored, packed codes and scale bytes, and dequantized in registers to exact 16-bit
//     floats (no BF16 panels in a workspace: a quarter of the bytes, and no expansion pass in front);
//   - the query heads that share a key / value head, and their few queries, are the 32 columns of ONE wave
//     (q_heads / kv_heads * Sq <= 32), so every K and V byte is read by one wave only;
//   - the keys are the parallelism: the key tiles are cut into `key_splits` contiguous ranges, one wave per (key / value
//     head, range), no barriers (LDS only as a wave's own staging space for V); each wave leaves its un-normalised
//     result, running maximum and sum in the workspace and a second kernel combines the ranges exactly:
//       m* = max_c m_c,   out = sum_c O_c 2^(m_c - m*) / sum_c l_c 2^(m_c - m*).
//     The probabilities of a range are cast against that range's own running maximum, so the result depends on
//     key_splits (with one range it is the other kernel's result up to summation order).
//
// Layouts in registers. First product, S^T[key, query] = K_tile . Q^T on v_mfma_f32_32x32x16_bf16: lane l of the A
// operand holds key l % 32 and 8 head dimensions, of the B operand query column l % 32 and the same 8 dimensions. Which
// 8 does not matter as long as both agree (a sum over the head dimension): lane half h = l / 32 reads the D / 4
// contiguous bytes of codes of dimensions (D / 2) h .. of its row, and k-step s multiplies word s of them, i.e.
// dimensions (D / 2) h + 8 s .. + 7, for K and Q alike. Second product, O^T[d, query] += V^T . P^T: the probabilities
// leave attention_tile.h as the B operand of two k-steps with the tile's keys in accumulator order
// (16 j + 4 h + {0,1,2,3,8,9,10,11}); lane (d, h) picks exactly those eight codes out of the 16 bytes its V^T row has
// for the tile: two 16-bit pieces of two words, one byte permute.
#include "../../include/amxfp4.h"
#include "attention_tile.h"
#include "dequant_regs.h"
#include "gemm_common.h"
#include "kernels.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// The 16-bit type the operands are dequantized to. FP8-E5M2 scales: FP16 with a bias of 2^-3 (every element * scale / 8
// lies in [2^-20, 43008] with at most 5 significant bits: an FP16 number, subnormals included; the scale byte is the
// upper byte of an FP16, so the dequantization is a conversion and one packed multiply); everything else: BF16.
template <int SCALE_KIND>
constexpr bool kDecodeF16 = SCALE_KIND == kScaleE5M2;

template <int SCALE_KIND>
__device__ __forceinline__ f32x16 decode_mfma(u32x4 a, u32x4 b, f32x16 acc) {
  if constexpr (kDecodeF16<SCALE_KIND>)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

// Eight codes (one word) of one group -> eight exact 16-bit floats (element * scale has at most 6 significant bits).
// FP8-E5M2 scales: FP16, biased (above). Power-of-two scales: the FP4 -> BF16 conversion applies the scale itself (it
// reads the exponent field of a float). FP8-E4M3 scales: FP32 decode, times the scale of the element's sign class as a
// float, truncated to BF16.
template <int SCALE_KIND, bool ASYM>
__device__ __forceinline__ u32x4 decode_word(uint32_t word, uint32_t byte_pos, uint32_t byte_neg) {
  u32x4 r;
  if constexpr (kDecodeF16<SCALE_KIND>) {
    const uint32_t sp = ((byte_pos << 8) | (byte_pos << 24)) & 0x7F007F00u, sn = ((byte_neg << 8) | (byte_neg << 24)) & 0x7F007F00u;
    r = u32x4{dequant2_f16<ASYM, 0>(word, sp, sn), dequant2_f16<ASYM, 1>(word, sp, sn),
              dequant2_f16<ASYM, 2>(word, sp, sn), dequant2_f16<ASYM, 3>(word, sp, sn)};
  } else if constexpr (SCALE_KIND == kScaleE8M0Floor || SCALE_KIND == kScaleE8M0Round) {
    const uint32_t sp = byte_pos << 23, sn = byte_neg << 23;
    r = u32x4{dequant2_pot<ASYM, 0>(word, sp, sn), dequant2_pot<ASYM, 1>(word, sp, sn),
              dequant2_pot<ASYM, 2>(word, sp, sn), dequant2_pot<ASYM, 3>(word, sp, sn)};
  } else {
    const uint32_t sp = f2u(scale_value<SCALE_KIND>(byte_pos)), sn = ASYM ? f2u(scale_value<SCALE_KIND>(byte_neg)) : sp;
    r = u32x4{dequant2_f32<ASYM, 0>(word, sp, sn), dequant2_f32<ASYM, 1>(word, sp, sn),
              dequant2_f32<ASYM, 2>(word, sp, sn), dequant2_f32<ASYM, 3>(word, sp, sn)};
  }
  return r;
}

// One row's share of a lane for the first product: the D / 4 bytes of codes of dimensions (D / 2) h .. and the scale
// bytes of their D / 64 groups (positive, negative; equal for symmetric formats).
template <int D>
struct RowPiece {
  uint32_t word[D / 16];
  uint32_t sp[D / 64], sn[D / 64];
};

template <int D, bool ASYM>
__device__ __forceinline__ void load_row_piece(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                               int64_t row, int h, RowPiece<D>& p) {
  const uint4* src = reinterpret_cast<const uint4*>(codes + row * (D / 2) + h * (D / 4));
#pragma unroll
  for (int i = 0; i < D / 64; ++i) {
    const uint4 c = src[i];
    p.word[4 * i] = c.x, p.word[4 * i + 1] = c.y, p.word[4 * i + 2] = c.z, p.word[4 * i + 3] = c.w;
    const int64_t g = row * (D / 32) + h * (D / 64) + i;
    if constexpr (ASYM) {
      const uint32_t pair = *reinterpret_cast<const uint16_t*>(scales + g * 2);
      p.sp[i] = pair & 255u, p.sn[i] = pair >> 8;
    } else {
      p.sp[i] = p.sn[i] = scales[g];
    }
  }
}

// A V^T row's share of a lane for one key tile: the 16 bytes of codes of the tile's 32 keys and the group's scales.
struct VPiece {
  uint4 codes;
  uint32_t sp, sn;
};

template <bool ASYM>
__device__ __forceinline__ void load_v_piece(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                             int64_t row, int64_t Sk, int t, VPiece& p) {
  p.codes = *reinterpret_cast<const uint4*>(codes + row * (Sk >> 1) + (int64_t)t * 16);
  const int64_t g = row * (Sk >> 5) + t;
  if constexpr (ASYM) {
    const uint32_t pair = *reinterpret_cast<const uint16_t*>(scales + g * 2);
    p.sp = pair & 255u, p.sn = pair >> 8;
  } else {
    p.sp = p.sn = scales[g];
  }
}

constexpr int kDecodeCols = 32;  // query columns of a wave

// grid: (key_splits, kv_heads); block: one wave. part: [kv_heads][32 columns][key_splits][D + 2] floats: the
// un-normalised O of the column in that range, then its running maximum (log2 units) and its sum; only the columns
// that hold a query are written.
//
// CHUNKED (Sk % 256 == 0): V^T rows are contiguous along the keys, so a key tile is 16 bytes of each of the D rows, one
// eighth of a cache line per row, and a wave that fetched them tile by tile would request every line of V eight times
// (and every line of V's scale bytes as often). The wave instead brings V in chunks of 8 key tiles: whole 128-byte
// lines of all D rows by direct-to-LDS loads (8 rows x 128 bytes per load; the 16-byte piece of tile j of row r goes to
// slot j ^ ((r >> 1) & 7) of the row's line in LDS, so that the 32 rows a tile read touches spread over the banks), and
// the chunk's scale bytes as D rows of 4-byte words. One chunk of LDS per wave, refilled when the wave has finished
// the previous chunk (its other wave on the SIMD works meanwhile); no barrier: a wave reads only what it loaded.
template <int SCALE_KIND, bool ASYM, int D, bool CHUNKED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attention_decode_kernel(
    const uint8_t* __restrict__ Qc, const uint8_t* __restrict__ Qs, const uint8_t* __restrict__ Kc,
    const uint8_t* __restrict__ Ks, const uint8_t* __restrict__ Vc, const uint8_t* __restrict__ Vs,
    float* __restrict__ part, int Sq, int Sk, int per, int tiles_per_split, float scale_log2, int causal) {
  constexpr int kSteps = D / 16, kRowBlocks = D / 32;
  constexpr int kScaleParts = ASYM ? 4 : 2;  // 4-byte words of scale bytes a row has per chunk of 8 tiles
  __shared__ __attribute__((aligned(1024))) uint8_t v_lines[CHUNKED ? D * 128 : 16];
  __shared__ __attribute__((aligned(256))) uint8_t v_scale_words[CHUNKED ? kScaleParts * D * 4 : 16];
  const int lane = threadIdx.x & 63, col = lane & 31, h = lane >> 5;
  const int split = (int)blockIdx.x, nsplits = (int)gridDim.x, g = (int)blockIdx.y;
  const int off = Sk - Sq;
  const bool col_valid = col < per * Sq;
  const int qi = col_valid ? col % Sq : 0;
  // a padding column multiplies zeros and sees every key: its numbers stay finite and are never read
  const int limit = col_valid && causal ? qi + off : Sk - 1;

  // this column's query as the B operand of the first product, resident in registers
  u32x4 qf[kSteps];
  if (col_valid) {
    RowPiece<D> q;
    load_row_piece<D, ASYM>(Qc, Qs, ((int64_t)g * per + col / Sq) * Sq + qi, h, q);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) qf[s] = decode_word<SCALE_KIND, ASYM>(q.word[s], q.sp[s >> 2], q.sn[s >> 2]);
  } else {
#pragma unroll
    for (int s = 0; s < kSteps; ++s) qf[s] = u32x4{0, 0, 0, 0};
  }
  // FP16 operands carry 2^-3 each: the scores come out divided by 2^6, the second product (probabilities times 2^8, so
  // that the smallest of them, 2^-17, is a normal FP16 number, times V / 8) multiplied by 2^5
  constexpr bool kF16 = kDecodeF16<SCALE_KIND>;
  const float score_scale = kF16 ? scale_log2 * 64.0f : scale_log2;

  f32x16 o[kRowBlocks];
#pragma unroll
  for (int db = 0; db < kRowBlocks; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m = -__builtin_inff(), l = 0.f;
  const int row_in_tile = 4 * h;  // key of accumulator register v: 8 (v / 4) + row_in_tile + v % 4

  const int tiles_all = Sk >> 5;
  const int t0 = split * tiles_per_split;
  const int t1 = t0 + tiles_per_split < tiles_all ? t0 + tiles_per_split : tiles_all;
  const int64_t krow0 = (int64_t)g * Sk + col;                      // K row of this lane in tile 0 (key = lane % 32)
  const int64_t vrow0 = (int64_t)g * D + col;                       // V^T row of this lane in row block 0
  // lane half h takes the low (h = 0) or high (h = 1) 16-bit pieces of two neighbouring words: keys 4 h .. 4 h + 3 and
  // 4 h + 8 .. 4 h + 11 of each 16
  const uint32_t pick = h ? 0x07060302u : 0x05040100u;

  // CHUNKED: this head's V^T codes and scale bytes as raw buffers (reads past the end return zeros), and the lane's
  // share of a load of 8 rows x 128 bytes: row L / 8 of the eight, the piece that belongs in slot L % 8
  const int v_row_bytes = Sk >> 1, vs_row_bytes = (Sk >> 5) * (ASYM ? 2 : 1);
  // (the addresses are the same in every lane; said explicitly, or the descriptors end up in vector registers and
  // every load in a loop over their distinct values)
  auto uniform_ptr = [](const uint8_t* p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return reinterpret_cast<uint8_t*>(((uint64_t)hi << 32) | lo);
  };
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(Vc + (int64_t)g * D * v_row_bytes), 0, __builtin_amdgcn_readfirstlane(D * v_row_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t vs_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(Vs + (int64_t)g * D * vs_row_bytes), 0, __builtin_amdgcn_readfirstlane(D * vs_row_bytes), 0x00020000);
  const int v_gather0 = (lane >> 3) * v_row_bytes + (((lane & 7) ^ (lane >> 4)) << 4);        // even load units
  const int v_gather1 = (lane >> 3) * v_row_bytes + (((lane & 7) ^ (4 + (lane >> 4))) << 4);  // odd load units
  const int v_read_swz = (col >> 1) & 7;  // rows 32 db + col: (row >> 1) & 7 does not depend on db

  RowPiece<D> kp;
  VPiece vp[CHUNKED ? 1 : kRowBlocks];
  if (t0 < t1) {
    load_row_piece<D, ASYM>(Kc, Ks, krow0 + (int64_t)t0 * 32, h, kp);
    if constexpr (!CHUNKED) {
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) load_v_piece<ASYM>(Vc, Vs, vrow0 + db * 32, Sk, t0, vp[db]);
    }
  }
  for (int t = t0; t < t1; ++t) {
    if constexpr (CHUNKED) {
      if (t == t0 || (t & 7) == 0) {
        // the wave is done with the previous chunk (its reads have returned): fetch the chunk of tile t
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int chunk = t >> 3;
#pragma unroll
        for (int u = 0; u < D / 8; ++u)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lds_ptr_t)(v_lines + u * 1024), 16,
                                                   (u & 1) ? v_gather1 : v_gather0,
                                                   u * 8 * v_row_bytes + chunk * 128, 0, 0);
#pragma unroll
        for (int q = 0; q < kScaleParts; ++q)
#pragma unroll
          for (int k = 0; k < D / 64; ++k)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(vs_rsrc, (lds_ptr_t)(v_scale_words + (q * D + 64 * k) * 4), 4,
                                                     lane * vs_row_bytes,
                                                     64 * k * vs_row_bytes + chunk * (kScaleParts * 4) + q * 4, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    }
    // the next tile's bytes are requested before this tile's arithmetic
    RowPiece<D> kn = kp;
    VPiece vn[CHUNKED ? 1 : kRowBlocks];
    if constexpr (!CHUNKED) {
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) vn[db] = vp[db];
    }
    if (t + 1 < t1) {
      load_row_piece<D, ASYM>(Kc, Ks, krow0 + (int64_t)(t + 1) * 32, h, kn);
      if constexpr (!CHUNKED) {
#pragma unroll
        for (int db = 0; db < kRowBlocks; ++db) load_v_piece<ASYM>(Vc, Vs, vrow0 + db * 32, Sk, t + 1, vn[db]);
      }
    }

    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < kSteps; ++ks) {
      const u32x4 a = decode_word<SCALE_KIND, ASYM>(kp.word[ks], kp.sp[ks >> 2], kp.sn[ks >> 2]);
      s = decode_mfma<SCALE_KIND>(a, qf[ks], s);
    }
    const bool masked = causal && t * 32 + 31 > off;  // some key of the tile is masked for the first query (uniform)
    AMX_ATTENTION_TILE_PROBS(true, s, score_scale, masked, t * 32 + row_in_tile, limit, m, l, pb, alpha, kF16)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // the maximum moved for some query: rescale
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const u32x4 b = {pb[4 * j], pb[4 * j + 1], pb[4 * j + 2], pb[4 * j + 3]};
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) {
        uint32_t w0, w1, vsp, vsn;
        if constexpr (CHUNKED) {
          // the tile's 16 bytes of V^T row 32 db + col, 8 of them per k-step, and the row's scale bytes for the tile
          const int tj = t & 7, row = db * 32 + col;
          const uint2 c = *reinterpret_cast<const uint2*>(v_lines + row * 128 + ((tj ^ v_read_swz) << 4) + 8 * j);
          w0 = c.x, w1 = c.y;
          if constexpr (ASYM) {
            const uint32_t pair = *reinterpret_cast<const uint16_t*>(v_scale_words + ((tj >> 1) * D + row) * 4 + (tj & 1) * 2);
            vsp = pair & 255u, vsn = pair >> 8;
          } else {
            vsp = vsn = v_scale_words[((tj >> 2) * D + row) * 4 + (tj & 3)];
          }
        } else {
          w0 = j ? vp[db].codes.z : vp[db].codes.x, w1 = j ? vp[db].codes.w : vp[db].codes.y;
          vsp = vp[db].sp, vsn = vp[db].sn;
        }
        const u32x4 a = decode_word<SCALE_KIND, ASYM>(__builtin_amdgcn_perm(w1, w0, pick), vsp, vsn);
        o[db] = decode_mfma<SCALE_KIND>(a, b, o[db]);
      }
    }
    kp = kn;
    if constexpr (!CHUNKED) {
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) vp[db] = vn[db];
    }
  }

  // register 4c + r of row block db is d = 32 db + 8 c + 4 h + r of column col
  if (!col_valid) return;
  float* dst = part + (((int64_t)g * kDecodeCols + col) * nsplits + split) * (D + 2);
  const float unbias = kF16 ? 0.03125f : 1.0f;  // 2^-5, exact
#pragma unroll
  for (int db = 0; db < kRowBlocks; ++db)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float* d4 = dst + db * 32 + c * 8 + 4 * h;
      d4[0] = o[db][4 * c] * unbias, d4[1] = o[db][4 * c + 1] * unbias, d4[2] = o[db][4 * c + 2] * unbias,
      d4[3] = o[db][4 * c + 3] * unbias;
    }
  if (h == 0) dst[D] = m, dst[D + 1] = l;
}

// One wave per (kv head, column that holds a query): the exact combination of the ranges, in FP32. The lanes first
// share out the ranges (maximum, then every range's weight 2^(m_c - m*), 0 for a range in which the query saw no key,
// and the weighted sum of the l_c), then the head dimensions (the ranges' rows are read whole lines at a time, eight
// ranges in flight).
constexpr int kDecodeMaxSplits = 1024;
template <int D>
__global__ __launch_bounds__(64) void attention_decode_combine_kernel(const float* __restrict__ part,
                                                                      float* __restrict__ out, int per, int Sq,
                                                                      int nsplits) {
  __shared__ float weight[kDecodeMaxSplits];
  const int lane = threadIdx.x, col = (int)blockIdx.x, g = (int)blockIdx.y;
  const float* base = part + ((int64_t)g * kDecodeCols + col) * nsplits * (D + 2);
  float mx = -__builtin_inff();
  for (int c = lane; c < nsplits; c += 64)
    if (base[(int64_t)c * (D + 2) + D + 1] > 0.f) mx = fmaxf(mx, base[(int64_t)c * (D + 2) + D]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
  float den = 0.f;
  for (int c = lane; c < nsplits; c += 64) {
    const float lc = base[(int64_t)c * (D + 2) + D + 1];
    const float w = lc > 0.f ? __builtin_amdgcn_exp2f(base[(int64_t)c * (D + 2) + D] - mx) : 0.f;
    weight[c] = w;
    den += w * lc;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) den += __shfl_xor(den, d, 64);
  __syncthreads();
  const float inv = 1.0f / den;
  float* dst = out + (((int64_t)g * per + col / Sq) * Sq + col % Sq) * D;
#pragma unroll
  for (int d = lane; d < D; d += 64) {
    float num = 0.f;
#pragma unroll 8
    for (int c = 0; c < nsplits; ++c) num += weight[c] * base[(int64_t)c * (D + 2) + d];
    dst[d] = num * inv;
  }
}

bool attention_decode_supported(int64_t Hq, int64_t Hkv, int64_t Sq, int64_t head_dim) {
  return Hkv > 0 && Hq % Hkv == 0 && (Hq / Hkv) * Sq <= kDecodeCols && (head_dim == 128 || head_dim == 64);
}

size_t attention_decode_workspace_bytes(int64_t Hkv, int64_t head_dim, int64_t key_splits) {
  return (size_t)(Hkv * key_splits * kDecodeCols * (head_dim + 2) * 4);
}

template <int SK, bool ASYM, int D>
static hipError_t launch_decode(int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk, const uint8_t* Qc, const uint8_t* Qs,
                                const uint8_t* Kc, const uint8_t* Ks, const uint8_t* Vc, const uint8_t* Vs, float scale,
                                int causal, int splits, float* out, float* part, hipStream_t s) {
  const int per = (int)(Hq / Hkv), tiles = (int)(Sk / 32), tiles_per_split = (tiles + splits - 1) / splits;
  // whole chunks of 8 key tiles, and V^T of one head within the 32-bit offsets of a buffer: V through LDS by chunks
  if (Sk % 256 == 0 && Sk <= (1 << 24))
    hipLaunchKernelGGL((attention_decode_kernel<SK, ASYM, D, true>), dim3((unsigned)splits, (unsigned)Hkv), dim3(64), 0, s,
                       Qc, Qs, Kc, Ks, Vc, Vs, part, (int)Sq, (int)Sk, per, tiles_per_split,
                       scale * 1.4426950408889634f, causal);
  else
    hipLaunchKernelGGL((attention_decode_kernel<SK, ASYM, D, false>), dim3((unsigned)splits, (unsigned)Hkv), dim3(64), 0, s,
                       Qc, Qs, Kc, Ks, Vc, Vs, part, (int)Sq, (int)Sk, per, tiles_per_split,
                       scale * 1.4426950408889634f, causal);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attention_decode_combine_kernel<D>), dim3((unsigned)(per * Sq), (unsigned)Hkv), dim3(64), 0, s, part,
                     out, per, (int)Sq, splits);
  return hipGetLastError();
}

hipError_t launch_attention_decode(int scale_kind, bool asym, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk,
                                   int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales,
                                   const uint8_t* K_codes, const uint8_t* K_scales, const uint8_t* V_codes,
                                   const uint8_t* V_scales, float scale, int causal, int key_splits, float* out,
                                   void* workspace, hipStream_t s) {
  float* part = reinterpret_cast<float*>(workspace);
  auto go = [&]<int SK, bool ASYM>() {
    if (head_dim == 128)
      return launch_decode<SK, ASYM, 128>(Hq, Hkv, Sq, Sk, Q_codes, Q_scales, K_codes, K_scales, V_codes, V_scales, scale,
                                          causal, key_splits, out, part, s);
    return launch_decode<SK, ASYM, 64>(Hq, Hkv, Sq, Sk, Q_codes, Q_scales, K_codes, K_scales, V_codes, V_scales, scale,
                                       causal, key_splits, out, part, s);
  };
  switch (scale_kind) {
    case kScaleE5M2: return asym ? go.template operator()<kScaleE5M2, true>() : go.template operator()<kScaleE5M2, false>();
    case kScaleE4M3: return asym ? go.template operator()<kScaleE4M3, true>() : go.template operator()<kScaleE4M3, false>();
    case kScaleE8M0Floor:
      return asym ? go.template operator()<kScaleE8M0Floor, true>() : go.template operator()<kScaleE8M0Floor, false>();
    case kScaleE8M0Round:
      return asym ? go.template operator()<kScaleE8M0Round, true>() : go.template operator()<kScaleE8M0Round, false>();
    default: return hipErrorInvalidValue;
  }
}

}  // namespace amx
