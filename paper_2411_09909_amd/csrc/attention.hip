// Fused quantized attention: out = softmax(scale * Q_hat . K_hat^T) . V_hat with both products on quantized operands
// (Sec. 5.1 quantizes Q.K^T and the attention map times V) and the attention map never written to memory: the scores
// of one tile of 32 keys become un-normalised probabilities against the running row maximum (online softmax), the
// tile of probabilities is cast as ONE group per query along the keys (the same element and scale format as the
// operands; FP32 values go into the cast), multiplied with the V tile, and the row sum divides at the end.
//
// Everything is computed transposed so that no data has to change lanes between the two products:
//   S^T[key, query] = K_tile[32 keys x D] . Q^T[D x 32 queries]      (MFMA 32x32x16 BF16, A = K rows, B = Q rows)
//   O^T[d, query]  += V^T[d x 32 keys]    . P^T[32 keys x 32 queries] (A = V^T, B = the probabilities)
// In a 32x32 accumulator lane l holds column l % 32 (one query) and rows 8c + 4(l/32) + r (c, r = 0..3) in register
// 4c + r: all 32 keys of a query sit in the two lanes l and l ^ 32, so the row maximum, the row sum and the group
// maximum of the cast are 16 in-lane steps and one exchange, and registers 8j .. 8j+7 of S^T, converted to BF16, are
// already the B operand of k-step j of the second product, provided V^T was staged with its keys in that order
// (expand_kernel<PERMUTE>). Workgroup = kAttnWaves waves x 32 queries; the K and V fragments of a key tile are brought into
// LDS once per workgroup by direct-to-LDS loads, double buffered.
#include "../../include/amxfp4.h"
#include "attention_tile.h"
#include "cast_math.h"
#include "gemm_common.h"

namespace amx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Waves per workgroup, 32 queries each. A wave's work on a tile is one long dependent chain (fragment reads -> eight
// chained MFMAs -> maximum, exponentials, sum, cast -> MFMAs), and the barrier of a workgroup keeps its waves in the
// same phase of it, so what hides the chain's latencies is waves of OTHER workgroups on the same SIMD: four waves per
// workgroup and a register budget of a third of the file put three workgroups on a compute unit (8 waves with two
// per SIMD: 0.243-0.248 ms for 32 heads x 4096; this: 0.229; a quarter of the file, four workgroups: 0.251, the heavy
// and light query blocks of a causal problem then all start at once).
constexpr int kAttnWaves = 4;
constexpr int kAttnQ = 32 * kAttnWaves;     // queries per workgroup

// kAttnD: the head dimension, 128 or 64. A key tile is kAttnD / 16 K fragments (one per 16 of D) and as many V^T
// fragments (D / 32 row blocks x 2 k-steps), dealt over the waves: wave w brings K and V fragments w, w + kAttnWaves,
// ... (with more waves than fragments the first ones would bring K, the others V).
template <int SCALE_KIND, int kAttnD>
__global__ __launch_bounds__(64 * kAttnWaves) __attribute__((amdgpu_waves_per_eu(3, 3))) void attention_fused_kernel(
    const uint16_t* __restrict__ Qp, const uint16_t* __restrict__ Kp, const uint16_t* __restrict__ Vp,
    float* __restrict__ out, int Sq, int Sk, int Sqp, int Skv, int kv_group, float scale_log2, int causal,
    int merged_bf16) {
  static_assert(kAttnD == 128 || kAttnD == 64, "head dimension");
  // FP8-E5M2 scales: the second product runs on FP16 operands. The cast leaves the probabilities as FP16 times 2^8
  // (the scale byte is the upper byte of an FP16: a conversion and a packed multiply per pair instead of a conversion,
  // two multiplies and a permute), V^T comes as an FP16 panel biased by 2^-3, and the 2^5 is taken out with the row
  // sum at the end. Same values, same sums.
  constexpr bool kPF16 = SCALE_KIND == kScaleE5M2;
  constexpr int kAttnKFrags = kAttnD / 16, kAttnVFrags = (kAttnD / 32) * 2;
  static_assert(kAttnKFrags == kAttnVFrags && (kAttnKFrags % kAttnWaves == 0 || 2 * kAttnKFrags == kAttnWaves),
                "fragments must divide over the waves");
  // two stages of (K tile, V tile), separate arrays so that loads into one stage are known not to alias reads of the
  // other
  __shared__ __attribute__((aligned(1024))) uint8_t ldsK0[kAttnKFrags * kFragBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsV0[kAttnVFrags * kFragBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsK1[kAttnKFrags * kFragBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t ldsV1[kAttnVFrags * kFragBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // Workgroups are dealt to the 8 XCDs round-robin by their linear id (x fastest). x walks the query heads, so every
  // XCD gets the same mix of light and heavy query blocks of a causal problem, and (when the head count is a multiple
  // of 8) a contiguous range of heads, i.e. heads that share a key/value head share an L2. y walks the query blocks,
  // last block first: under a causal mask those have the most key tiles and should start first.
  const int nheads = (int)gridDim.x;
  const int h = (nheads & 7) == 0 ? (int)(blockIdx.x & 7) * (nheads >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const int g = h / kv_group;
  const int qblock = (int)(gridDim.y - 1 - blockIdx.y);
  const int q0 = qblock * kAttnQ, qw = q0 + wave * 32;
  const int off = Sk - Sq;  // causal: query i sees keys <= i + off
  const bool wave_active = qw < Sqp;

  // key tiles this workgroup / this wave walks over (uniform)
  const int tiles_all = Sk / 32;
  const int last_q_block = (q0 + kAttnQ < Sqp ? q0 + kAttnQ : Sqp) - 1;
  const int nt = causal ? min(tiles_all, (last_q_block + off) / 32 + 1) : tiles_all;
  const int nt_wave = !wave_active ? 0 : (causal ? min(tiles_all, (qw + 31 + off) / 32 + 1) : tiles_all);

  // K panel of this key/value head: tile t = 8 contiguous fragments; V^T panel: 4 row blocks of Skv / 16 fragments
  // (Skv = Sk rounded up to the panel's K granularity of 64). Raw buffers: reads past the end return zero.
  const int64_t kfrags_head = (int64_t)tiles_all * kAttnKFrags, vfrags_head = (int64_t)(kAttnD / 32) * (Skv / 16);
  const uint8_t* Kbase = reinterpret_cast<const uint8_t*>(Kp) + g * kfrags_head * kFragBytes;
  const uint8_t* Vbase = reinterpret_cast<const uint8_t*>(Vp) + g * vfrags_head * kFragBytes;
  const __amdgpu_buffer_rsrc_t Kr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(Kbase), 0, (int)(kfrags_head * kFragBytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t Vr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(Vbase), 0, (int)(vfrags_head * kFragBytes), 0x00020000);
  const int lane_off = lane * 16;

  // wave w brings K fragments w, w + kAttnWaves, .. and the V fragments of the same numbers (V fragment f = row block
  // f / 2, k-step f % 2) of tile T into stage (DK, DV)
#define AMX_ATTN_LOAD(T, DK, DV)                                                                                   \
  do {                                                                                                             \
    if constexpr (kAttnKFrags >= kAttnWaves) {                                                                     \
      _Pragma("unroll") for (int i_ = 0; i_ < kAttnKFrags / kAttnWaves; ++i_) {                                    \
        const int f_ = wave + kAttnWaves * i_;                                                                     \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(Kr, (lds_ptr_t)((DK) + f_ * kFragBytes), 16, lane_off,            \
                                                 ((T) * kAttnKFrags + f_) * kFragBytes, 0, 0);                     \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(Vr, (lds_ptr_t)((DV) + f_ * kFragBytes), 16, lane_off,            \
                                                 ((f_ >> 1) * (Skv / 16) + (f_ & 1) + 2 * (T)) * kFragBytes, 0, 0);\
      }                                                                                                            \
    } else if (wave < kAttnKFrags) { /* uniform over the wave */                                                   \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Kr, (lds_ptr_t)((DK) + wave * kFragBytes), 16, lane_off,            \
                                               ((T) * kAttnKFrags + wave) * kFragBytes, 0, 0);                     \
    } else {                                                                                                       \
      const int f_ = wave - kAttnKFrags;                                                                           \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Vr, (lds_ptr_t)((DV) + f_ * kFragBytes), 16, lane_off,              \
                                               ((f_ >> 1) * (Skv / 16) + (f_ & 1) + 2 * (T)) * kFragBytes, 0, 0);  \
    }                                                                                                              \
  } while (0)

  // this wave's 32 queries as the B operand of the first product: 8 k-steps over D, resident in registers
  bf16x8 qf[kAttnKFrags];
  if (wave_active) {
    const uint8_t* qsrc = reinterpret_cast<const uint8_t*>(Qp) +
                          (((int64_t)h * (Sqp / 32) + qw / 32) * kAttnKFrags) * kFragBytes + lane_off;
#pragma unroll
    for (int kb = 0; kb < kAttnKFrags; ++kb) qf[kb] = *reinterpret_cast<const bf16x8*>(qsrc + kb * kFragBytes);
  } else {
#pragma unroll
    for (int kb = 0; kb < kAttnKFrags; ++kb) qf[kb] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
  }

  f32x16 o[kAttnD / 32];
#pragma unroll
  for (int db = 0; db < kAttnD / 32; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m = -__builtin_inff(), l = 0.f;  // running maximum (scaled score, in units of log2) and sum of this lane's query
  const int limit = causal ? qw + (lane & 31) + off : Sk - 1;  // last key this lane's query may attend to
  const int row_in_tile = 4 * (lane >> 5);                    // key of register v: 8 (v / 4) + row_in_tile + v % 4

  // One key tile from stage (CK, CV).
#define AMX_ATTN_TILE(T, CK, CV)                                                                                   \
  if ((T) < nt_wave) {                                                                                             \
    f32x16 s;                                                                                                      \
    _Pragma("unroll") for (int v = 0; v < 16; ++v) s[v] = 0.f;                                                     \
    _Pragma("unroll") for (int kb = 0; kb < kAttnKFrags; ++kb) {                                                   \
      const bf16x8 a = *reinterpret_cast<const bf16x8*>((CK) + kb * kFragBytes + lane_off);                        \
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kb], s, 0, 0, 0);                                          \
    }                                                                                                              \
    const bool diagonal = causal && (T) * 32 + 31 > qw + off; /* some key of the tile is masked for some query */ \
    AMX_ATTENTION_TILE_PROBS(false, s, scale_log2, diagonal, (T) * 32 + row_in_tile, limit, m, l, pb, alpha, kPF16)       \
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) { /* the maximum moved for some query: rescale */        \
      _Pragma("unroll") for (int db = 0; db < kAttnD / 32; ++db)                                                   \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) o[db][v] *= alpha;                                          \
    }                                                                                                              \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                                                \
      const u32x4 b = {pb[4 * j], pb[4 * j + 1], pb[4 * j + 2], pb[4 * j + 3]};                                    \
      _Pragma("unroll") for (int db = 0; db < kAttnD / 32; ++db) {                                                 \
        const u32x4 a = *reinterpret_cast<const u32x4*>((CV) + (db * 2 + j) * kFragBytes + lane_off);              \
        if constexpr (kPF16)                                                                                       \
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), \
                                                         o[db], 0, 0, 0);                                          \
        else                                                                                                       \
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),                           \
                                                          __builtin_bit_cast(bf16x8, b), o[db], 0, 0, 0);          \
      }                                                                                                            \
    }                                                                                                              \
  }

  // prologue: tile 0 into stage 0
  AMX_ATTN_LOAD(0, ldsK0, ldsV0);
  AMX_WAIT_VMCNT(0);
  AMX_BARRIER();
  for (int t = 0; t < nt; t += 2) {
    // stage 1 was last read during tile t - 1; the barrier that ended it lets every wave refill it now
    if (t + 1 < nt) AMX_ATTN_LOAD(t + 1, ldsK1, ldsV1);
    AMX_ATTN_TILE(t, ldsK0, ldsV0);
    AMX_WAIT_VMCNT(0);
    AMX_BARRIER();
    if (t + 1 < nt) {  // uniform over the workgroup
      if (t + 2 < nt) AMX_ATTN_LOAD(t + 2, ldsK0, ldsV0);
      AMX_ATTN_TILE(t + 1, ldsK1, ldsV1);
      AMX_WAIT_VMCNT(0);
      AMX_BARRIER();
    }
  }
#undef AMX_ATTN_TILE
#undef AMX_ATTN_LOAD

  // out[h][query][d] = O^T[d][query] / l; register 4c + r of row block db is d = 32 db + 8 c + 4 (lane / 32) + r.
  // merged_bf16: the same values rounded to BF16 and written token-major, out[query][h * D + d] (the layout the output
  // projection's cast reads: no head-merge pass over an FP32 copy).
  const int q = qw + (lane & 31);
  if (wave_active && q < Sq && merged_bf16) {
    const float inv = (kPF16 ? 0.03125f : 1.0f) / l;
    uint16_t* dst = reinterpret_cast<uint16_t*>(out) + ((int64_t)q * nheads + h) * kAttnD + row_in_tile;
#pragma unroll
    for (int db = 0; db < kAttnD / 32; ++db)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        *reinterpret_cast<uint2*>(dst + db * 32 + c * 8) = make_uint2(
            pack2(o[db][4 * c] * inv, o[db][4 * c + 1] * inv), pack2(o[db][4 * c + 2] * inv, o[db][4 * c + 3] * inv));
  } else if (wave_active && q < Sq) {
    const float inv = (kPF16 ? 0.03125f : 1.0f) / l;
    float* dst = out + ((int64_t)h * Sq + q) * kAttnD + row_in_tile;
#pragma unroll
    for (int db = 0; db < kAttnD / 32; ++db)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 v4 = make_float4(o[db][4 * c] * inv, o[db][4 * c + 1] * inv, o[db][4 * c + 2] * inv,
                                      o[db][4 * c + 3] * inv);
        *reinterpret_cast<float4*>(dst + db * 32 + c * 8) = v4;
      }
  }
}

size_t attention_workspace_bytes(int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk, int64_t head_dim) {
  return (size_t)((Hq * round_up(Sq, 32) + Hkv * Sk + Hkv * round_up(Sk, 64)) * head_dim * 2);
}

template <int SK, int kAttnD>
static hipError_t launch_attn(const uint16_t* Qp, const uint16_t* Kp, const uint16_t* Vp, float* out, int64_t Hq,
                              int64_t Hkv, int64_t Sq, int64_t Sk, float scale, int causal, int merged_bf16,
                              hipStream_t s) {
  const int64_t Sqp = round_up(Sq, 32);
  const dim3 grid((unsigned)Hq, (unsigned)((Sqp + kAttnQ - 1) / kAttnQ));
  hipLaunchKernelGGL((attention_fused_kernel<SK, kAttnD>), grid, dim3(64 * kAttnWaves), 0, s, Qp, Kp, Vp, out, (int)Sq,
                     (int)Sk, (int)Sqp, (int)round_up(Sk, 64), (int)(Hq / Hkv), scale * 1.4426950408889634f, causal,
                     merged_bf16);
  return hipGetLastError();
}

template <int kAttnD>
static hipError_t launch_attention_fused_d(int scale_kind, bool asym, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk,
                                  const uint8_t* Q_codes, const uint8_t* Q_scales, const uint8_t* K_codes,
                                  const uint8_t* K_scales, const uint8_t* V_codes, const uint8_t* V_scales, float scale,
                                  int causal, float* out, bool merged_bf16, void* workspace, hipStream_t s,
                                  const KernelTimer& timer) {
  const int64_t Sqp = round_up(Sq, 32);
  uint16_t* Qp = reinterpret_cast<uint16_t*>(workspace);
  uint16_t* Kp = Qp + Hq * Sqp * kAttnD;
  uint16_t* Vp = Kp + Hkv * Sk * kAttnD;
  // Q, K: rows = tokens, K = head dimension; V^T: rows = head dimension, K = keys, in the accumulator's key order
  hipError_t e = launch_expand_bf16(scale_kind, asym, 32, Q_codes, Q_scales, Sq, kAttnD, Sqp, kAttnD, Hq, false, Qp, s);
  if (e != hipSuccess) return e;
  e = launch_expand_bf16(scale_kind, asym, 32, K_codes, K_scales, Sk, kAttnD, Sk, kAttnD, Hkv, false, Kp, s);
  if (e != hipSuccess) return e;
  e = launch_expand_bf16(scale_kind, asym, 32, V_codes, V_scales, kAttnD, Sk, kAttnD, round_up(Sk, 64), Hkv, true, Vp, s);
  if (e != hipSuccess) return e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  switch (scale_kind) {
    case kScaleE5M2: e = launch_attn<kScaleE5M2, kAttnD>(Qp, Kp, Vp, out, Hq, Hkv, Sq, Sk, scale, causal, merged_bf16, s); break;
    case kScaleE4M3: e = launch_attn<kScaleE4M3, kAttnD>(Qp, Kp, Vp, out, Hq, Hkv, Sq, Sk, scale, causal, merged_bf16, s); break;
    case kScaleE8M0Floor: e = launch_attn<kScaleE8M0Floor, kAttnD>(Qp, Kp, Vp, out, Hq, Hkv, Sq, Sk, scale, causal, merged_bf16, s); break;
    case kScaleE8M0Round: e = launch_attn<kScaleE8M0Round, kAttnD>(Qp, Kp, Vp, out, Hq, Hkv, Sq, Sk, scale, causal, merged_bf16, s); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

hipError_t launch_attention_fused(int scale_kind, bool asym, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk,
                                  int64_t head_dim, const uint8_t* Q_codes, const uint8_t* Q_scales,
                                  const uint8_t* K_codes, const uint8_t* K_scales, const uint8_t* V_codes,
                                  const uint8_t* V_scales, float scale, int causal, float* out, bool merged_bf16,
                                  void* workspace, hipStream_t s, const KernelTimer& timer) {
  if (head_dim == 128)
    return launch_attention_fused_d<128>(scale_kind, asym, Hq, Hkv, Sq, Sk, Q_codes, Q_scales, K_codes, K_scales, V_codes,
                                         V_scales, scale, causal, out, merged_bf16, workspace, s, timer);
  if (head_dim == 64)
    return launch_attention_fused_d<64>(scale_kind, asym, Hq, Hkv, Sq, Sk, Q_codes, Q_scales, K_codes, K_scales, V_codes,
                                        V_scales, scale, causal, out, merged_bf16, workspace, s, timer);
  return hipErrorInvalidValue;
}

}  // namespace amx
