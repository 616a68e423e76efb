// Fused quantized attention for FEW queries against many keys (decoding: one or a handful of new tokens against a long
// key / value cache). Same per-tile arithmetic as attention.hip (Sec. 5.1 quantizes Q.K^T and the attention map times V;
// online softmax over key tiles of 32, each tile of probabilities cast as one group per query), but organised for the
// shape: the work is reading K and V once, so
//   - K and V are read as they are stored, packed codes and scale bytes, and dequantized in registers to exact BF16
//     (no BF16 panels in a workspace: a quarter of the bytes, and no expansion pass in front);
//   - the query heads that share a key / value head, and their few queries, are the 32 columns of ONE wave
//     (q_heads / kv_heads * Sq <= 32), so every K and V byte is read by one wave only;
//   - the keys are the parallelism: the key tiles are cut into `key_splits` contiguous ranges, one wave per (key / value
//     head, range), no LDS and no barriers; each wave leaves its un-normalised result, running maximum and sum in the
//     workspace and a second kernel combines the ranges exactly:
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

// Eight codes (one word) of one group -> eight BF16, for any scale format: FP32 decode, times the scale of the
// element's sign class as a float, truncated to BF16 (exact: at most 6 significant bits).
template <int SCALE_KIND, bool ASYM>
__device__ __forceinline__ bf16x8 decode_word(uint32_t word, uint32_t byte_pos, uint32_t byte_neg) {
  const uint32_t sp = f2u(scale_value<SCALE_KIND>(byte_pos)), sn = ASYM ? f2u(scale_value<SCALE_KIND>(byte_neg)) : sp;
  const u32x4 r = {dequant2_f32<ASYM, 0>(word, sp, sn), dequant2_f32<ASYM, 1>(word, sp, sn),
                   dequant2_f32<ASYM, 2>(word, sp, sn), dequant2_f32<ASYM, 3>(word, sp, sn)};
  return __builtin_bit_cast(bf16x8, r);
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

// grid: (key_splits, kv_heads); block: one wave. part: [kv_heads][key_splits][32 columns][D + 2] floats: the
// un-normalised O of the column, then its running maximum (log2 units) and its sum.
template <int SCALE_KIND, bool ASYM, int D>
__global__ __launch_bounds__(64) void attention_decode_kernel(
    const uint8_t* __restrict__ Qc, const uint8_t* __restrict__ Qs, const uint8_t* __restrict__ Kc,
    const uint8_t* __restrict__ Ks, const uint8_t* __restrict__ Vc, const uint8_t* __restrict__ Vs,
    float* __restrict__ part, int Sq, int Sk, int per, int tiles_per_split, float scale_log2, int causal) {
  constexpr int kSteps = D / 16, kRowBlocks = D / 32;
  const int lane = threadIdx.x & 63, col = lane & 31, h = lane >> 5;
  const int split = (int)blockIdx.x, nsplits = (int)gridDim.x, g = (int)blockIdx.y;
  const int off = Sk - Sq;
  const bool col_valid = col < per * Sq;
  const int qi = col_valid ? col % Sq : 0;
  // a padding column multiplies zeros and sees every key: its numbers stay finite and are never read
  const int limit = col_valid && causal ? qi + off : Sk - 1;

  // this column's query as the B operand of the first product, resident in registers
  bf16x8 qf[kSteps];
  if (col_valid) {
    RowPiece<D> q;
    load_row_piece<D, ASYM>(Qc, Qs, ((int64_t)g * per + col / Sq) * Sq + qi, h, q);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) qf[s] = decode_word<SCALE_KIND, ASYM>(q.word[s], q.sp[s >> 2], q.sn[s >> 2]);
  } else {
#pragma unroll
    for (int s = 0; s < kSteps; ++s) qf[s] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
  }

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

  RowPiece<D> kp;
  VPiece vp[kRowBlocks];
  if (t0 < t1) {
    load_row_piece<D, ASYM>(Kc, Ks, krow0 + (int64_t)t0 * 32, h, kp);
#pragma unroll
    for (int db = 0; db < kRowBlocks; ++db) load_v_piece<ASYM>(Vc, Vs, vrow0 + db * 32, Sk, t0, vp[db]);
  }
  for (int t = t0; t < t1; ++t) {
    // the next tile's bytes are requested before this tile's arithmetic
    RowPiece<D> kn = kp;
    VPiece vn[kRowBlocks];
#pragma unroll
    for (int db = 0; db < kRowBlocks; ++db) vn[db] = vp[db];
    if (t + 1 < t1) {
      load_row_piece<D, ASYM>(Kc, Ks, krow0 + (int64_t)(t + 1) * 32, h, kn);
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) load_v_piece<ASYM>(Vc, Vs, vrow0 + db * 32, Sk, t + 1, vn[db]);
    }

    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < kSteps; ++ks) {
      const bf16x8 a = decode_word<SCALE_KIND, ASYM>(kp.word[ks], kp.sp[ks >> 2], kp.sn[ks >> 2]);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s, 0, 0, 0);
    }
    const bool masked = causal && t * 32 + 31 > off;  // some key of the tile is masked for the first query (uniform)
    AMX_ATTENTION_TILE_PROBS(true, s, scale_log2, masked, t * 32 + row_in_tile, limit, m, l, pb, alpha)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // the maximum moved for some query: rescale
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{pb[4 * j], pb[4 * j + 1], pb[4 * j + 2], pb[4 * j + 3]});
#pragma unroll
      for (int db = 0; db < kRowBlocks; ++db) {
        const uint32_t w0 = j ? vp[db].codes.z : vp[db].codes.x, w1 = j ? vp[db].codes.w : vp[db].codes.y;
        const bf16x8 a = decode_word<SCALE_KIND, ASYM>(__builtin_amdgcn_perm(w1, w0, pick), vp[db].sp, vp[db].sn);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o[db], 0, 0, 0);
      }
    }
    kp = kn;
#pragma unroll
    for (int db = 0; db < kRowBlocks; ++db) vp[db] = vn[db];
  }

  // register 4c + r of row block db is d = 32 db + 8 c + 4 h + r of column col
  float* dst = part + (((int64_t)g * nsplits + split) * kDecodeCols + col) * (D + 2);
#pragma unroll
  for (int db = 0; db < kRowBlocks; ++db)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float* d4 = dst + db * 32 + c * 8 + 4 * h;
      d4[0] = o[db][4 * c], d4[1] = o[db][4 * c + 1], d4[2] = o[db][4 * c + 2], d4[3] = o[db][4 * c + 3];
    }
  if (h == 0) dst[D] = m, dst[D + 1] = l;
}

// One thread per (kv head, valid column, 4 head dimensions): the exact combination of the ranges, in FP32.
template <int D>
__global__ __launch_bounds__(256) void attention_decode_combine_kernel(const float* __restrict__ part,
                                                                       float* __restrict__ out, int kv_heads, int per,
                                                                       int Sq, int nsplits) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cols = per * Sq;
  if (idx >= (int64_t)kv_heads * cols * (D / 4)) return;
  const int d4 = (int)(idx % (D / 4));
  const int col = (int)((idx / (D / 4)) % cols);
  const int g = (int)(idx / ((int64_t)(D / 4) * cols));
  const float* base = part + ((int64_t)g * nsplits * kDecodeCols + col) * (D + 2);
  const int64_t stride = (int64_t)kDecodeCols * (D + 2);
  float mx = -__builtin_inff();
  for (int c = 0; c < nsplits; ++c)
    if (base[c * stride + D + 1] > 0.f) mx = fmaxf(mx, base[c * stride + D]);
  float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
  for (int c = 0; c < nsplits; ++c) {
    const float lc = base[c * stride + D + 1];
    if (!(lc > 0.f)) continue;  // a range in which this query saw no key
    const float w = __builtin_amdgcn_exp2f(base[c * stride + D] - mx);
    den += w * lc;
#pragma unroll
    for (int e = 0; e < 4; ++e) num[e] += w * base[c * stride + 4 * d4 + e];
  }
  const float inv = 1.0f / den;
  float* dst = out + (((int64_t)g * per + col / Sq) * Sq + col % Sq) * D + 4 * d4;
  *reinterpret_cast<float4*>(dst) = make_float4(num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv);
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
  hipLaunchKernelGGL((attention_decode_kernel<SK, ASYM, D>), dim3((unsigned)splits, (unsigned)Hkv), dim3(64), 0, s, Qc, Qs,
                     Kc, Ks, Vc, Vs, part, (int)Sq, (int)Sk, per, tiles_per_split, scale * 1.4426950408889634f, causal);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t threads = Hkv * per * Sq * (D / 4);
  hipLaunchKernelGGL((attention_decode_combine_kernel<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, part,
                     out, (int)Hkv, per, (int)Sq, splits);
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
