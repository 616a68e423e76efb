// Fully quantized GEMM for FP8-E5M2 shared scales (the paper's AMXFP4, Sec. 4.2-4.3, and its symmetric "MXFP4") with
// the dequantization fused into the kernel: the packed E2M1 codes and the scale bytes travel HBM -> L2 -> LDS as they
// are (4.5 bits per element), are expanded to exact FP16 inside the workgroup and multiplied on the FP16 MFMA
// (v_mfma_f32_32x32x16_f16, FP32 accumulate). Compared with expanding into BF16 panels in a separate pass
// (gemm_bf16.hip) this moves 3.5x fewer bytes through the L2, which is what bounds that kernel, and needs no workspace.
//
// Exactness. A dequantized element is elem * S with elem in +-{0,.5,1,1.5,2,3,4,6} and S an E5M2 value: at most 5
// significant bits. An E5M2 byte is the high byte of an IEEE half, so S is an FP16 number as it stands. The kernel
// forms (elem * 2^-3) * S in packed FP16: v_cvt_scalef32_pk_f16_fp4 converts two codes and applies the power-of-two
// 2^-3, v_pk_mul_f16 multiplies by the scale of each element's own sign (Eq. 1), picked per 16-bit half with
// v_pk_ashrrev_i16 + v_bfi_b32. With the 2^-3 bias every representable product lies in [2^-20, 43008], inside the
// FP16 range including subnormals (which both the packed multiply and the MFMA honour), so no product is rounded.
// The bias of both operands is undone exactly by scaling the accumulators by 2^6 before they are stored.
//
// Structure (fused kernel). 512 threads = 8 waves compute a 256 x 256 tile: wave w multiplies row half w / 4 and
// column quarter w % 4 (4 x 2 MFMA tiles of 32x32) and expands rows of A (waves 0-3) or of B (waves 4-7); two waves
// share a SIMD, so one wave's expansion runs under the other's MFMAs.
//   raw ring  2 x 36 KiB: one stage = a K slice of 128: codes of the 256 A rows and 256 B rows (64 bytes per row,
//             staged in 16-row x 64-byte direct-to-LDS loads, chunk-permuted for conflict-free reads) + scale bytes.
//   expanded  2 x 32 KiB: one K slice of 32 as MFMA operand fragments (1 KiB = 64 lanes x 8 halves).
// Per K slice q every lane expands one group (32 codes) of its row of slice q+1 from the raw stage into the other
// fragment buffer while the wave multiplies slice q; the two are interleaved instruction by instruction. One barrier
// per slice; a raw stage is refilled four slices before it is needed. A second kernel further down (hybrid) takes A
// from an FP16 panel instead and expands only B.
#include "device_formats.h"
#include "gemm_common.h"

namespace amx {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr int kE5Tile = 256;            // tile edge (rows of A and of B per workgroup)
constexpr int kRawCodes = kE5Tile * 64;  // bytes of one operand's codes per raw stage (K = 128)

// The expansion of 8 codes (one dword w) into 8 halves is split into three phases that are issued behind three
// consecutive MFMAs, so that no instruction waits for the one just before it:
//   convert  r[i] = (two codes of byte i) * 2^-3 as packed FP16                       (v_cvt_scalef32_pk_f16_fp4)
//   select   s[i] = per half, the negative scale where r[i] < 0, else the positive one (v_pk_ashrrev_i16 + v_bfi_b32)
//   scale    out[i] = r[i] * s[i]                                                      (v_pk_mul_f16)
// select is written as the two instructions meant: the compiler otherwise lowers the idiom to compares and selects.
__device__ __forceinline__ void expand_convert(uint32_t w, uint32_t (&r)[4]) {
  r[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 0.125f, 0));
  r[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 0.125f, 1));
  r[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 0.125f, 2));
  r[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 0.125f, 3));
}
__device__ __forceinline__ void expand_sign_mask(const uint32_t (&r)[4], uint32_t (&m)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) asm("v_pk_ashrrev_i16 %0, %1, %2" : "=v"(m[i]) : "s"(0x000F000Fu), "v"(r[i]));
}
__device__ __forceinline__ void expand_select(uint32_t (&m)[4], uint32_t sp2, uint32_t sn2) {
#pragma unroll
  for (int i = 0; i < 4; ++i) asm("v_bfi_b32 %0, %0, %1, %2" : "+v"(m[i]) : "v"(sn2), "v"(sp2));
}
__device__ __forceinline__ uint4 expand_scale(const uint32_t (&r)[4], const uint32_t (&s)[4]) {
  uint32_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    o[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, r[i]) * __builtin_bit_cast(f16x2, s[i]));
  return make_uint4(o[0], o[1], o[2], o[3]);
}
__device__ __forceinline__ uint4 expand_scale1(const uint32_t (&r)[4], uint32_t s) {
  uint32_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    o[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, r[i]) * __builtin_bit_cast(f16x2, s));
  return make_uint4(o[0], o[1], o[2], o[3]);
}

template <bool ASYM>
__global__ __launch_bounds__(512) void gemm_e5m2_kernel(const uint8_t* __restrict__ Ac, const uint8_t* __restrict__ As,
                                                        const uint8_t* __restrict__ Bc, const uint8_t* __restrict__ Bs,
                                                        float* __restrict__ C, int64_t M, int64_t N, int64_t K,
                                                        int64_t ldc, int tiles_m, int tiles_n, int super_m) {
  constexpr int kScaleRow = ASYM ? 8 : 4;             // scale bytes per row per raw stage (4 groups)
  constexpr int kRawScales = kE5Tile * kScaleRow;     // per operand
  constexpr int kRawBytes = 2 * kRawCodes + 2 * kRawScales;
  constexpr int kExpHalf = (kE5Tile / 32) * 2 * kFragBytes;  // one operand: 8 row blocks x 2 k blocks x 1 KiB
  constexpr int kExpBytes = 2 * kExpHalf;
  constexpr int FM = 4, FN = 2;
  // separate arrays, so that the compiler can tell direct-to-LDS loads into one from reads of another
  __shared__ __attribute__((aligned(1024))) uint8_t raw0[kRawBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t raw1[kRawBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t exp0[kExpBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t exp1[kExpBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;  // wm also selects the operand this wave expands (0: A rows, 1: B rows)
  const int64_t b = blockIdx.z;
  int tm, tn;
  if (!tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, super_m, tm, tn)) return;  // uniform, before any barrier

  const int row_bytes = (int)(K >> 1);
  const int srow_bytes = (int)(K >> 5) * (ASYM ? 2 : 1);
  const int rows_a = (int)(M - (int64_t)tm * kE5Tile < kE5Tile ? M - (int64_t)tm * kE5Tile : kE5Tile);
  const int rows_b = (int)(N - (int64_t)tn * kE5Tile < kE5Tile ? N - (int64_t)tn * kE5Tile : kE5Tile);
  // raw buffers (stride 0): reads past the tile's last valid row return zero = code 0 / scale 0 = value 0
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Ac + (b * M + (int64_t)tm * kE5Tile) * row_bytes), 0, rows_a * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bc + (b * N + (int64_t)tn * kE5Tile) * row_bytes), 0, rows_b * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Asr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(As + (b * M + (int64_t)tm * kE5Tile) * srow_bytes), 0, rows_a * srow_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bs + (b * N + (int64_t)tn * kE5Tile) * srow_bytes), 0, rows_b * srow_bytes, 0x00020000);

  // ---- staging (direct-to-LDS loads), per wave and raw stage: 2 A-code + 2 B-code loads of 16 rows x 64 bytes, and
  // scale loads of 4 bytes per lane (asymmetric: 32 rows x 8 bytes, one for A and one for B per wave; symmetric:
  // 64 rows x 4 bytes, waves 0-3 fetch A's, waves 4-7 B's).
  const int cgather = (lane >> 2) * row_bytes + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);
  const int sgather = ASYM ? (lane >> 1) * srow_bytes + (lane & 1) * 4 : lane * srow_bytes;
#define AMX_ISSUE_RAW(ST, DST)                                                                                        \
  {                                                                                                                   \
    _Pragma("unroll") for (int l = 0; l < 2; ++l) {                                                                   \
      const int h_ = wave + 8 * l; /* half row block (16 rows) 0..15 */                                               \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + h_ * 1024), 16, cgather,                       \
                                               h_ * 16 * row_bytes + (ST) * 64, 0, 0);                                \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)((DST) + kRawCodes + h_ * 1024), 16, cgather,           \
                                               h_ * 16 * row_bytes + (ST) * 64, 0, 0);                                \
    }                                                                                                                 \
    if constexpr (ASYM) {                                                                                             \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Asr, (lds_ptr_t)((DST) + 2 * kRawCodes + wave * 256), 4, sgather,      \
                                               wave * 32 * srow_bytes + (ST) * 8, 0, 0);                              \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Bsr, (lds_ptr_t)((DST) + 2 * kRawCodes + kRawScales + wave * 256), 4,  \
                                               sgather, wave * 32 * srow_bytes + (ST) * 8, 0, 0);                     \
    } else {                                                                                                          \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wm ? Bsr : Asr,                                                        \
                                               (lds_ptr_t)((DST) + 2 * kRawCodes + wm * kRawScales + wn * 256), 4,    \
                                               sgather, wn * 64 * srow_bytes + (ST) * 4, 0, 0);                       \
    }                                                                                                                 \
  }

  // ---- expansion: lane tid owns row tid % 256 of the operand its wave expands (waves 0-3: A, waves 4-7: B). The raw
  // codes and scale bytes of a K slice are read into registers one slice ahead (AMX_RAW_READ); the AMX_EXPAND_PH*
  // macros turn them into fragment chunks (8 halves) and write those into the fragment buffer.
  const int xrow = tid & 255;
  const int xcodes = wm * kRawCodes + xrow * 64;
  const int xswz = (xrow >> 2) & 3;
  const int xscales = 2 * kRawCodes + wm * kRawScales + xrow * kScaleRow;
  // destination: fragment (row block, k block) = 1 KiB; 16-byte slot (k half * 32 + row % 32) inside it
  const int xdst = wm * kExpHalf + (xrow >> 5) * 2 * kFragBytes + (xrow & 31) * 16;
  uint32_t wq[4], sq = 0;    // codes / scale bytes of the slice being expanded
  uint32_t wnx[4], snx = 0;  // ... of the slice after it (prefetched)
  uint32_t sp2 = 0, sn2 = 0;
#define AMX_RAW_READ(CHUNK, SRC)                                                                  \
  {                                                                                               \
    const uint4 w_ = *reinterpret_cast<const uint4*>((SRC) + xcodes + (((CHUNK) ^ xswz) << 4));   \
    wnx[0] = w_.x, wnx[1] = w_.y, wnx[2] = w_.z, wnx[3] = w_.w;                                   \
    if constexpr (ASYM)                                                                           \
      snx = *reinterpret_cast<const uint16_t*>((SRC) + xscales + (CHUNK) * 2);                    \
    else                                                                                          \
      snx = *reinterpret_cast<const uint8_t*>((SRC) + xscales + (CHUNK));                         \
  }
#define AMX_RAW_ADVANCE()                                                                          \
  {                                                                                                \
    wq[0] = wnx[0], wq[1] = wnx[1], wq[2] = wnx[2], wq[3] = wnx[3], sq = snx;                      \
    sp2 = __builtin_amdgcn_perm(0u, sq, 0x000c000cu); /* (S_p, S_p) as FP16: byte << 8 per half */ \
    if constexpr (ASYM) sn2 = __builtin_amdgcn_perm(0u, sq, 0x010c010cu);                          \
  }
  // expansion of chunk D (codes 8D .. 8D+7: k block D / 2, k half D % 2) of the group, in the three phases
  uint32_t xr[4], xs[4];
#define AMX_EXPAND_PH0(D)                         \
  {                                               \
    expand_convert(wq[D], xr);                    \
    if constexpr (ASYM) expand_sign_mask(xr, xs); \
  }
#define AMX_EXPAND_PH1(D) \
  { if constexpr (ASYM) expand_select(xs, sp2, sn2); }
#define AMX_EXPAND_PH2(D, DST)                                                                    \
  {                                                                                               \
    uint4 o_;                                                                                     \
    if constexpr (ASYM) o_ = expand_scale(xr, xs); else o_ = expand_scale1(xr, sp2);              \
    *reinterpret_cast<uint4*>((DST) + xdst + ((D) >> 1) * kFragBytes + ((D) & 1) * 512) = o_;     \
  }
#define AMX_EXPAND_CHUNK(D, DST) \
  {                              \
    AMX_EXPAND_PH0(D);           \
    AMX_EXPAND_PH1(D);           \
    AMX_EXPAND_PH2(D, DST);      \
  }

  // ---- multiplication: 16 MFMAs per wave and K slice, number T = 8 * k block + 2 * i + j
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int moffA = (wm * FM) * 2 * kFragBytes + lane * 16;
  const int moffB = kExpHalf + (wn * FN) * 2 * kFragBytes + lane * 16;
  f16x8 fa[2][FM], fb[2][FN];  // [k block][row block]
#pragma unroll
  for (int e = 0; e < 8; ++e) {  // k block 1 registers start as zeros: the first slice's "previous slice" MFMAs add 0
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[1][i][e] = (_Float16)0;
#pragma unroll
    for (int j = 0; j < FN; ++j) fb[1][j][e] = (_Float16)0;
  }
#define AMX_FRAG_READ(KB, SRC)                                                                                        \
  {                                                                                                                   \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) fb[KB][j] =                                                        \
        *reinterpret_cast<const f16x8*>((SRC) + moffB + (j * 2 + (KB)) * kFragBytes);                                 \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) fa[KB][i] =                                                        \
        *reinterpret_cast<const f16x8*>((SRC) + moffA + (i * 2 + (KB)) * kFragBytes);                                 \
  }
#define AMX_MFMA(T)                                                                     \
  acc[((T) >> 1) & 3][(T) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(                \
      fa[(T) >> 3][((T) >> 1) & 3], fb[(T) >> 3][(T) & 1], acc[((T) >> 1) & 3][(T) & 1], 0, 0, 0)

  // One K slice q = 16 MFMA slots per wave (two waves share each SIMD, so 32 per matrix pipe). At the top: wait for this
  // wave's LDS traffic of the previous slice (and, when VM is set, its direct-to-LDS loads) and meet the other waves;
  // ISSUE (may be empty) refills a raw stage that is dead by now. Then the k block 0 fragments of this slice and the
  // raw data of slice q+2 are requested. Slots 0..7 run the k block 1 MFMAs of the PREVIOUS slice (operands still in
  // registers), which covers the barrier skew and the latency of those reads; slots 8..15 run this slice's k block 0
  // MFMAs, after its k block 1 fragments have been requested. The 4 chunks of slice q+1 are expanded in slots 0..11,
  // one phase per slot (convert, select, scale + write to XDST), so every LDS write is long complete at the next barrier.
  // XDST receives slice q+1, MSRC holds slice q, (PCHUNK, PSRC) is the raw data of slice q+2.
#define AMX_SLICE(VM, ISSUE, PCHUNK, PSRC, XDST, MSRC)                                      \
  {                                                                                         \
    __builtin_amdgcn_s_waitcnt((VM) ? 0x0070 : 0xC07F); /* lgkmcnt(0) [+ vmcnt(0)] */       \
    AMX_BARRIER();                                                                          \
    ISSUE;                                                                                  \
    AMX_FRAG_READ(0, MSRC);                                                                 \
    AMX_RAW_ADVANCE();                                                                      \
    AMX_RAW_READ(PCHUNK, PSRC);                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                      \
    _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                        \
      if (t == 8) AMX_FRAG_READ(1, MSRC);                                                   \
      if (t < 8) {                                                                          \
        AMX_MFMA(8 + t);                                                                    \
      } else {                                                                              \
        AMX_MFMA(t - 8);                                                                    \
      }                                                                                     \
      if (t < 12) {                                                                         \
        if (t % 3 == 0) AMX_EXPAND_PH0(t / 3);                                              \
        if (t % 3 == 1) AMX_EXPAND_PH1(t / 3);                                              \
        if (t % 3 == 2) AMX_EXPAND_PH2(t / 3, XDST);                                        \
      }                                                                                     \
      __builtin_amdgcn_sched_barrier(0);                                                    \
    }                                                                                       \
  }

  // Raw stage R in CUR (the next one in NXT): slices 4R .. 4R+3 are multiplied, slices 4R+1 .. 4R+4 expanded from raw
  // data read one slice earlier. From the third slice on CUR is dead (its last chunk sits in registers), so the stage
  // after next is fetched into it there; that slice's barrier is also where the fetch of NXT, issued four slices ago,
  // is waited for. Past the end of K, fetch and expansion are pointed at the last real stage instead of being skipped;
  // their results are never multiplied.
#define AMX_STAGE(R, CUR, NXT)                                                                                   \
  {                                                                                                              \
    const int fetch_ = (R) + 2 < nstages ? (R) + 2 : nstages - 1;                                                \
    AMX_SLICE(0, , 2, CUR, exp1, exp0);                                                                          \
    AMX_SLICE(0, , 3, CUR, exp0, exp1);                                                                          \
    AMX_SLICE(1, AMX_ISSUE_RAW(fetch_, CUR), 0, NXT, exp1, exp0);                                                \
    AMX_SLICE(0, , 1, NXT, exp0, exp1);                                                                          \
  }

  const int nstages = (int)(K >> 7);
  AMX_ISSUE_RAW(0, raw0);
  AMX_ISSUE_RAW(nstages > 1 ? 1 : 0, raw1);
  __builtin_amdgcn_s_waitcnt(0x0070);
  AMX_BARRIER();
  // slice 0 is expanded up front; the raw data of slice 1 is left in the prefetch registers
  AMX_RAW_READ(0, raw0);
  AMX_RAW_ADVANCE();
  AMX_RAW_READ(1, raw0);
#pragma unroll
  for (int d = 0; d < 4; ++d) AMX_EXPAND_CHUNK(d, exp0);
  // (no branch inside the loop body: a conditional second stage makes the register allocator spill)
  int r = 0;
  for (; r + 2 <= nstages; r += 2) {
    AMX_STAGE(r, raw0, raw1);
    AMX_STAGE(r + 1, raw1, raw0);
  }
  if (r < nstages) AMX_STAGE(r, raw0, raw1);
#pragma unroll
  for (int t = 8; t < 16; ++t) AMX_MFMA(t);  // the last slice's deferred k block 1 MFMAs
  __builtin_amdgcn_s_waitcnt(0x0070);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_MFMA
#undef AMX_STAGE
#undef AMX_SLICE
#undef AMX_FRAG_READ
#undef AMX_EXPAND_CHUNK
#undef AMX_EXPAND_PH2
#undef AMX_EXPAND_PH1
#undef AMX_EXPAND_PH0
#undef AMX_RAW_ADVANCE
#undef AMX_RAW_READ
#undef AMX_ISSUE_RAW

  store_c_tiles<FM, FN, 6 /* 2^6 undoes the operand bias */>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * kE5Tile + wm * FM * 32,
                        (int64_t)tn * kE5Tile + wn * FN * 32);
}

bool e5m2_fused_supported(int64_t M, int64_t N, int64_t K) {
  // K in whole raw stages; per-tile byte offsets must fit the 32-bit buffer offsets
  return K % 128 == 0 && K <= (1 << 22) && M > 0 && N > 0;
}

hipError_t launch_gemm_e5m2_fused(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                  const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                  int64_t ldc, int64_t batch, hipStream_t s, const KernelTimer& timer) {
  const int tiles_m = (int)((M + kE5Tile - 1) / kE5Tile), tiles_n = (int)((N + kE5Tile - 1) / kE5Tile);
  int super_m;
  const dim3 grid(supertile_grid(tiles_m, tiles_n, super_m), 1, (unsigned)batch);
  hipError_t e;
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  if (asym)
    hipLaunchKernelGGL((gemm_e5m2_kernel<true>), grid, dim3(512), 0, s, A_codes, A_scales, B_codes, B_scales, C, M, N,
                       K, ldc, tiles_m, tiles_n, super_m);
  else
    hipLaunchKernelGGL((gemm_e5m2_kernel<false>), grid, dim3(512), 0, s, A_codes, A_scales, B_codes, B_scales, C, M, N,
                       K, ldc, tiles_m, tiles_n, super_m);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

// ------------------------------------------------------------------------------------------------ hybrid ----------
// A from a panel, B dequantized in the kernel. The activations (A) are expanded once per call into an FP16
// fragment-major panel (gemm_bf16.hip's layout, values biased by 2^-3) and staged by linear direct-to-LDS copies; the
// weights (B), the large operand, travel as packed codes + scale bytes and are expanded inside the workgroup exactly as
// in the kernel above. Per K slice of 32 a compute unit then pulls 16 KiB (A fragments) + 4.5 KiB (B codes and scales)
// through its vector cache instead of 32 KiB, which is what bounds the two-panel kernel, and each lane expands one
// group of one B row, half the work of the fully fused kernel. No expansion pass and no workspace for B.
//
// 256 threads = 2 x 2 waves, each 4 x 4 MFMA tiles. LDS: A ring 4 x 16 KiB (one K slice each), raw B ring 2 x 18 KiB
// (K = 128 each), expanded B 2 x 16 KiB. Slice q (8 steps of 4 MFMAs): multiplies slice q (A fragments read from the
// ring two steps ahead, B fragments of the whole slice already in registers), reads the B fragments of slice q+1 into
// the other register set, expands slice q+2 (raw data in registers) into the fragment buffer that slice q's fragments
// came from, reads the raw data of slice q+3 into registers, and issues the A loads of slice q+3.
template <bool ASYM>
__global__ __launch_bounds__(256) void gemm_e5m2_hybrid_kernel(const uint16_t* __restrict__ Ap,
                                                               const uint8_t* __restrict__ Bc,
                                                               const uint8_t* __restrict__ Bs, float* __restrict__ C,
                                                               int64_t M, int64_t N, int64_t Mp, int64_t K, int64_t ldc,
                                                               int tiles_m, int tiles_n, int super_m) {
  constexpr int kScaleRow = ASYM ? 8 : 4;          // scale bytes per row per raw stage (4 groups)
  constexpr int kRawBytes = kRawCodes + kE5Tile * kScaleRow;
  constexpr int kStageA = (kE5Tile / 32) * 2 * kFragBytes;  // 8 row blocks x 2 k blocks x 1 KiB
  constexpr int kExpBytes = kStageA;                        // the same for B
  constexpr int FM = 4, FN = 4;
  constexpr int kRawLoads = ASYM ? 6 : 5;  // direct-to-LDS loads per wave and raw stage
  __shared__ __attribute__((aligned(1024))) uint8_t a0[kStageA];
  __shared__ __attribute__((aligned(1024))) uint8_t a1[kStageA];
  __shared__ __attribute__((aligned(1024))) uint8_t a2[kStageA];
  __shared__ __attribute__((aligned(1024))) uint8_t a3[kStageA];
  __shared__ __attribute__((aligned(1024))) uint8_t raw0[kRawBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t raw1[kRawBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t exp0[kExpBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t exp1[kExpBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t b = blockIdx.z;
  int tm, tn;
  if (!tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, super_m, tm, tn)) return;  // uniform, before any barrier

  const int kblocks = (int)(K >> 4);
  const int row_bytes = (int)(K >> 1);
  const int srow_bytes = (int)(K >> 5) * (ASYM ? 2 : 1);
  const int rows_b = (int)(N - (int64_t)tn * kE5Tile < kE5Tile ? N - (int64_t)tn * kE5Tile : kE5Tile);
  const __amdgpu_buffer_rsrc_t Ar = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(Ap) +
                           ((b * (Mp >> 5) + (int64_t)tm * (kE5Tile / 32)) * kblocks) * kFragBytes),
      0, (kE5Tile / 32) * kblocks * kFragBytes, 0x00020000);
  // raw buffers (stride 0): reads past the tile's last valid row return zero = code 0 / scale 0 = value 0
  const __amdgpu_buffer_rsrc_t Br = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bc + (b * N + (int64_t)tn * kE5Tile) * row_bytes), 0, rows_b * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t Bsr = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(Bs + (b * N + (int64_t)tn * kE5Tile) * srow_bytes), 0, rows_b * srow_bytes, 0x00020000);
  const int lane_off = lane * 16;

  // ---- staging. A: load L (0..3) of this wave for slice ST: fragment f = wave + 4 L (row block f / 2, k block f % 2).
  // B, per raw stage: 4 code loads of 16 rows x 64 bytes per wave (chunk-permuted for conflict-free reads) and scale
  // loads of 4 bytes per lane (asymmetric: 32 rows x 8 bytes, 2 per wave; symmetric: 64 rows x 4 bytes, 1 per wave).
#define AMX_ISSUE_A(L, ST, DST)                                                                                   \
  {                                                                                                               \
    const int f_ = wave + 4 * (L);                                                                                \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(Ar, (lds_ptr_t)((DST) + f_ * kFragBytes), 16, lane_off,              \
                                             ((f_ >> 1) * kblocks + (ST) * 2 + (f_ & 1)) * kFragBytes, 0, 0);     \
  }
  const int cgather = (lane >> 2) * row_bytes + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);
  const int sgather = ASYM ? (lane >> 1) * srow_bytes + (lane & 1) * 4 : lane * srow_bytes;
#define AMX_ISSUE_RAW(ST, DST)                                                                                    \
  {                                                                                                               \
    _Pragma("unroll") for (int l = 0; l < 4; ++l) {                                                               \
      const int h_ = wave + 4 * l; /* half row block (16 rows) 0..15 */                                           \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Br, (lds_ptr_t)((DST) + h_ * 1024), 16, cgather,                   \
                                               h_ * 16 * row_bytes + (ST) * 64, 0, 0);                            \
    }                                                                                                             \
    if constexpr (ASYM) {                                                                                         \
      _Pragma("unroll") for (int l = 0; l < 2; ++l) {                                                             \
        const int g_ = wave + 4 * l; /* 32 rows each */                                                           \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(Bsr, (lds_ptr_t)((DST) + kRawCodes + g_ * 256), 4, sgather,      \
                                                 g_ * 32 * srow_bytes + (ST) * 8, 0, 0);                          \
      }                                                                                                           \
    } else {                                                                                                      \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(Bsr, (lds_ptr_t)((DST) + kRawCodes + wave * 256), 4, sgather,      \
                                               wave * 64 * srow_bytes + (ST) * 4, 0, 0);                          \
    }                                                                                                             \
  }

  // ---- expansion: lane tid owns B row tid of the tile
  const int xrow = tid;
  const int xcodes = xrow * 64;
  const int xswz = (xrow >> 2) & 3;
  const int xscales = kRawCodes + xrow * kScaleRow;
  // destination: fragment (row block, k block) = 1 KiB; 16-byte slot (k half * 32 + row % 32) inside it
  const int xdst = (xrow >> 5) * 2 * kFragBytes + (xrow & 31) * 16;
  uint32_t wq[4], sq = 0;    // codes / scale bytes of the slice being expanded
  uint32_t wnx[4], snx = 0;  // ... of the slice after it (prefetched)
  uint32_t sp2 = 0, sn2 = 0;
#define AMX_RAW_READ(CHUNK, SRC)                                                                  \
  {                                                                                               \
    const uint4 w_ = *reinterpret_cast<const uint4*>((SRC) + xcodes + (((CHUNK) ^ xswz) << 4));   \
    wnx[0] = w_.x, wnx[1] = w_.y, wnx[2] = w_.z, wnx[3] = w_.w;                                   \
    if constexpr (ASYM)                                                                           \
      snx = *reinterpret_cast<const uint16_t*>((SRC) + xscales + (CHUNK) * 2);                    \
    else                                                                                          \
      snx = *reinterpret_cast<const uint8_t*>((SRC) + xscales + (CHUNK));                         \
  }
#define AMX_RAW_ADVANCE()                                                                          \
  {                                                                                                \
    wq[0] = wnx[0], wq[1] = wnx[1], wq[2] = wnx[2], wq[3] = wnx[3], sq = snx;                      \
    sp2 = __builtin_amdgcn_perm(0u, sq, 0x000c000cu); /* (S_p, S_p) as FP16: byte << 8 per half */ \
    if constexpr (ASYM) sn2 = __builtin_amdgcn_perm(0u, sq, 0x010c010cu);                          \
  }
  // expansion of chunk D (codes 8D .. 8D+7: k block D / 2, k half D % 2) of the group, in the three phases
  uint32_t xr[4], xs[4];
#define AMX_EXPAND_PH0(D)                         \
  {                                               \
    expand_convert(wq[D], xr);                    \
    if constexpr (ASYM) expand_sign_mask(xr, xs); \
  }
#define AMX_EXPAND_PH1(D) \
  { if constexpr (ASYM) expand_select(xs, sp2, sn2); }
#define AMX_EXPAND_PH2(D, DST)                                                                    \
  {                                                                                               \
    uint4 o_;                                                                                     \
    if constexpr (ASYM) o_ = expand_scale(xr, xs); else o_ = expand_scale1(xr, sp2);              \
    *reinterpret_cast<uint4*>((DST) + xdst + ((D) >> 1) * kFragBytes + ((D) & 1) * 512) = o_;     \
  }

  // ---- multiplication
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int offA = lane_off + (wm * FM) * 2 * kFragBytes;
  const int offB = lane_off + (wn * FN) * 2 * kFragBytes;
  f16x8 aR[4];         // A fragment of step t in aR[t & 3], read two steps ahead
  f16x8 bS[2][2][FN];  // [slice parity][k block][column block]
#define AMX_READ_B(SET, Q8, SRC) \
  bS[SET][(Q8) >> 2][(Q8) & 3] = *reinterpret_cast<const f16x8*>((SRC) + offB + (((Q8) & 3) * 2 + ((Q8) >> 2)) * kFragBytes)

  const int nslices = (int)(K >> 5), nraw = (int)(K >> 7);
  // One slice. At the top: this wave's LDS traffic of the previous slice is complete and its direct-to-LDS loads up to
  // the A fragments of slice Q+1 have landed (VMC = number of loads issued after those: the 4 A loads of the previous
  // slice, plus the raw loads if that slice issued them); then the barrier makes both true for the whole workgroup.
  // ISSUE (may be empty) refills a raw stage that is dead by now; it comes before this slice's A loads.
  // SET = Q % 2; XDST receives slice Q+2 (it held slice Q, whose fragments are in registers); FSRC holds slice Q+1;
  // (PCHUNK, PSRC) is the raw data of slice Q+3; CUR / NXT / FETCH are the A ring slots of slices Q, Q+1 and Q+3.
#define AMX_SLICE(Q, SET, VMC, ISSUE, PCHUNK, PSRC, XDST, FSRC, CUR, NXT, FETCH)                                    \
  {                                                                                                                 \
    __builtin_amdgcn_s_waitcnt(0x0070 | ((VMC) & 15) | (((VMC) >> 4) << 14)); /* vmcnt(VMC), lgkmcnt(0) */          \
    AMX_BARRIER();                                                                                                  \
    const int fetch_ = (Q) + 3 < nslices ? (Q) + 3 : nslices - 1;                                                   \
    ISSUE;                                                                                                          \
    AMX_RAW_ADVANCE();                                                                                              \
    AMX_RAW_READ(PCHUNK, PSRC);                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                              \
    _Pragma("unroll") for (int t = 0; t < 8; ++t) {                                                                 \
      {                                                                                                             \
        const int t2 = t + 2, ks2 = (t2 >> 2) & 1, i2 = t2 & 3;                                                     \
        const uint8_t* src_ = t2 < 8 ? (CUR) : (NXT);                                                               \
        aR[t2 & 3] = *reinterpret_cast<const f16x8*>(src_ + offA + (i2 * 2 + ks2) * kFragBytes);                    \
      }                                                                                                             \
      AMX_READ_B((SET) ^ 1, t, FSRC);                                                                               \
      if (t < 4) AMX_ISSUE_A(t, fetch_, FETCH);                                                                     \
      _Pragma("unroll") for (int p = 0; p < 12; ++p) {                                                              \
        if (p * 2 / 3 == t) {                                                                                       \
          if (p % 3 == 0) AMX_EXPAND_PH0(p / 3);                                                                    \
          if (p % 3 == 1) AMX_EXPAND_PH1(p / 3);                                                                    \
          if (p % 3 == 2) AMX_EXPAND_PH2(p / 3, XDST);                                                              \
        }                                                                                                           \
      }                                                                                                             \
      _Pragma("unroll") for (int j = 0; j < FN; ++j) acc[t & 3][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(        \
          aR[t & 3], bS[SET][t >> 2][j], acc[t & 3][j], 0, 0, 0);                                                   \
      __builtin_amdgcn_sched_barrier(0);                                                                            \
    }                                                                                                               \
  }
  // Raw stage R in RC (the next one in RN) covers slices 4R .. 4R+3. Slice 4R reads the stage's last chunk, so from
  // slice 4R+1 on RC is dead and the stage after next is fetched into it there. Past the end of K, fetches and
  // expansion are pointed at the last real stage / slice instead of being skipped; their results are never used.
#define AMX_STAGE(R, RC, RN)                                                                                        \
  {                                                                                                                 \
    const int rfetch_ = (R) + 2 < nraw ? (R) + 2 : nraw - 1;                                                        \
    AMX_SLICE(4 * (R), 0, 4, , 3, RC, exp0, exp1, a0, a1, a3);                                                      \
    AMX_SLICE(4 * (R) + 1, 1, 4, AMX_ISSUE_RAW(rfetch_, RC), 0, RN, exp1, exp0, a1, a2, a0);                        \
    AMX_SLICE(4 * (R) + 2, 0, 4 + kRawLoads, , 1, RN, exp0, exp1, a2, a3, a1);                                      \
    AMX_SLICE(4 * (R) + 3, 1, 4, , 2, RN, exp1, exp0, a3, a0, a2);                                                  \
  }

  // prologue: A slices 0..2 and raw stages 0, 1 in flight; slices 0 and 1 of B are expanded up front, the raw data of
  // slice 2 is left in the prefetch registers, the B fragments of slice 0 and the first A fragments in registers
  AMX_ISSUE_RAW(0, raw0);
  AMX_ISSUE_RAW(nraw > 1 ? 1 : 0, raw1);
#pragma unroll
  for (int l = 0; l < 4; ++l) AMX_ISSUE_A(l, 0, a0);
#pragma unroll
  for (int l = 0; l < 4; ++l) AMX_ISSUE_A(l, 1, a1);
#pragma unroll
  for (int l = 0; l < 4; ++l) AMX_ISSUE_A(l, 2, a2);
  __builtin_amdgcn_s_waitcnt(0x0070);  // everything
  AMX_BARRIER();
  AMX_RAW_READ(0, raw0);
  AMX_RAW_ADVANCE();
  AMX_RAW_READ(1, raw0);
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    AMX_EXPAND_PH0(d);
    AMX_EXPAND_PH1(d);
    AMX_EXPAND_PH2(d, exp0);
  }
  AMX_RAW_ADVANCE();
  AMX_RAW_READ(2, raw0);
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    AMX_EXPAND_PH0(d);
    AMX_EXPAND_PH1(d);
    AMX_EXPAND_PH2(d, exp1);
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's fragment writes
  AMX_BARRIER();
#pragma unroll
  for (int q8 = 0; q8 < 8; ++q8) AMX_READ_B(0, q8, exp0);
  aR[0] = *reinterpret_cast<const f16x8*>(a0 + offA);
  aR[1] = *reinterpret_cast<const f16x8*>(a0 + offA + 2 * kFragBytes);

  // (no branch inside the loop body: a conditional second stage makes the register allocator spill)
  int r = 0;
  for (; r + 2 <= nraw; r += 2) {
    AMX_STAGE(r, raw0, raw1);
    AMX_STAGE(r + 1, raw1, raw0);
  }
  if (r < nraw) AMX_STAGE(r, raw0, raw1);
  __builtin_amdgcn_s_waitcnt(0x0070);  // nothing may still be writing this workgroup's LDS when it retires
#undef AMX_STAGE
#undef AMX_SLICE
#undef AMX_READ_B
#undef AMX_EXPAND_PH2
#undef AMX_EXPAND_PH1
#undef AMX_EXPAND_PH0
#undef AMX_RAW_ADVANCE
#undef AMX_RAW_READ
#undef AMX_ISSUE_RAW
#undef AMX_ISSUE_A

  store_c_tiles<FM, FN, 6 /* 2^6 undoes the operand bias */>(acc, C + b * M * ldc, M, N, ldc, (int64_t)tm * kE5Tile + wm * FM * 32,
                        (int64_t)tn * kE5Tile + wn * FN * 32);
}

bool e5m2_hybrid_supported(int64_t M, int64_t N, int64_t K) {
  // K in whole raw stages; per-tile byte offsets must fit the 32-bit buffer offsets
  return K % 128 == 0 && K <= (1 << 22) && M > 0 && N > 0;
}

size_t e5m2_hybrid_workspace_bytes(int64_t M, int64_t K, int64_t batch) {
  return (size_t)(batch * round_up(M, kE5Tile) * K * 2);
}

hipError_t launch_gemm_e5m2_hybrid(bool asym, int64_t M, int64_t N, int64_t K, const uint8_t* A_codes,
                                   const uint8_t* A_scales, const uint8_t* B_codes, const uint8_t* B_scales, float* C,
                                   int64_t ldc, int64_t batch, void* workspace, hipStream_t s,
                                   const KernelTimer& timer) {
  const int64_t Mp = round_up(M, kE5Tile);
  uint16_t* Ap = reinterpret_cast<uint16_t*>(workspace);
  hipError_t e = launch_expand_f16_e5m2(asym, A_codes, A_scales, M, K, Mp, K, batch, Ap, s);
  if (e != hipSuccess) return e;
  const int tiles_m = (int)((M + kE5Tile - 1) / kE5Tile), tiles_n = (int)((N + kE5Tile - 1) / kE5Tile);
  int super_m;
  const dim3 grid(supertile_grid(tiles_m, tiles_n, super_m), 1, (unsigned)batch);
  if (timer.start && (e = hipEventRecord(timer.start, s)) != hipSuccess) return e;
  if (asym)
    hipLaunchKernelGGL((gemm_e5m2_hybrid_kernel<true>), grid, dim3(256), 0, s, Ap, B_codes, B_scales, C, M, N, Mp, K,
                       ldc, tiles_m, tiles_n, super_m);
  else
    hipLaunchKernelGGL((gemm_e5m2_hybrid_kernel<false>), grid, dim3(256), 0, s, Ap, B_codes, B_scales, C, M, N, Mp, K,
                       ldc, tiles_m, tiles_n, super_m);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (timer.stop) e = hipEventRecord(timer.stop, s);
  return e;
}

}  // namespace amx
