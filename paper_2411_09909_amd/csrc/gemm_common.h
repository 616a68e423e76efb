// Pieces shared by the GEMM kernels: tile configuration, the 4-stage LDS ring bookkeeping, the XCD-aware tile order and
// the wait / barrier primitives of the software pipeline.
//
// Pipeline (both kernels): a workgroup tile of (32*FM*WM) x (32*FN*WN) outputs is computed by WM x WN waves, each
// owning FM x FN MFMA tiles of 32x32. K is consumed in stages; one stage holds, per 32-row block of either operand,
// 2 fragments of 1 KiB (64 lanes x 16 bytes = the register image of one MFMA operand). Four stage buffers form a
// ring: while stage S is multiplied, stage S+1 is already complete in LDS (fragment reads run ahead into it), and
// stages S+2 and S+3 are in flight as direct-to-LDS buffer loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "layer_math.h"

namespace amx {

constexpr int kFragBytes = 1024;  // one MFMA operand fragment: 64 lanes x 16 bytes

template <int WM, int WN, int FM, int FN>
struct TileCfg {
  static constexpr int kWaves = WM * WN;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kTileM = 32 * FM * WM;
  static constexpr int kTileN = 32 * FN * WN;
  static constexpr int kFragsA = (kTileM / 32) * 2;  // fragments per stage
  static constexpr int kFragsB = (kTileN / 32) * 2;
  static constexpr int kLoads = (kFragsA + kFragsB) / kWaves;  // direct-to-LDS loads per wave per stage
  static constexpr int kStageBytes = (kFragsA + kFragsB) * kFragBytes;
  static_assert(kFragsA % kWaves == 0 && kFragsB % kWaves == 0, "fragments must divide evenly over the waves");
  static_assert(FM % 2 == 0, "the A register ring of 4 needs an even number of steps per k-step");
};

// Supertile: the tiles that run at the same time on one XCD (32 CUs, one L2): 8 along M x 4 along N, so that every
// staged A panel is shared by 4 and every B panel by 8 workgroups through that L2. Workgroups are dealt to the 8 XCDs
// round-robin by their linear id, hence id % 8 picks the XCD and id / 8 the slot on it.
constexpr int kSuperM = 8, kSuperN = 4;

// Tile coordinates of workgroup `p`; false if it has no tile (grid padding).
__device__ __forceinline__ bool tile_of_workgroup(int p, int tiles_m, int tiles_n, int super_m, int& tm, int& tn) {
  const int xcd = p & 7, q = p >> 3;
  const int st = (q / (kSuperM * kSuperN)) * 8 + xcd, slot = q % (kSuperM * kSuperN);
  tm = (st % super_m) * kSuperM + slot % kSuperM;
  tn = (st / super_m) * kSuperN + slot / kSuperM;
  return tm < tiles_m && tn < tiles_n;
}

// Grid size (x) for a tiles_m x tiles_n problem: supertiles are dealt 8 at a time, one per XCD.
inline unsigned supertile_grid(int tiles_m, int tiles_n, int& super_m) {
  super_m = (tiles_m + kSuperM - 1) / kSuperM;
  const int super_n = (tiles_n + kSuperN - 1) / kSuperN;
  const int rounds = (super_m * super_n + 7) / 8;
  return (unsigned)(rounds * 8 * kSuperM * kSuperN);
}

// s_waitcnt immediate that waits until at most n (< 64) vector-memory operations are outstanding and nothing else
// (gfx9 encoding: vmcnt = bits 3:0 and 15:14, expcnt = bits 6:4, lgkmcnt = bits 11:8)
#define AMX_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// workgroup barrier without the memory fence __syncthreads() implies: the data movement around it is ordered by the
// explicit vmcnt waits (direct-to-LDS loads) and by the MFMA operand dependencies (LDS reads)
#define AMX_BARRIER() asm volatile("s_barrier" ::: "memory")

typedef __attribute__((address_space(3))) void* lds_ptr_t;

typedef float f32x16 __attribute__((ext_vector_type(16)));  // accumulator of one 32x32 MFMA tile

// Stores a wave's FM x FN accumulator tiles of 32x32 into C (row-major, leading dimension ldc), multiplied by
// 2^SCALE_LOG2 (0, or the power of two that undoes an operand bias) and, with ALPHA, by the run-time factor alpha.
// row_base / col_base: first row / column of the wave's tiles.
// Accumulator register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its tile. Rows >= M and columns
// >= N (partial tiles) are not written. Non-temporal stores: C is not read again by the kernel.
// Addressing: one raw buffer over the wave's window of C, from its first element to the last valid element of its last
// valid row. The row of a store is a scalar offset (a compile-time multiple of the row pitch), the column and the lane
// half's row offset a per-lane offset computed once per column tile, so a store costs one scalar addition; the hardware
// drops whatever falls beyond the window (the range check covers the scalar offset too: probed), which takes care of
// the rows >= M, and lanes whose column is >= N are given an offset beyond any window. Needs ldc <= 2^22 (the entry
// points check it): 128 rows of that pitch stay below 2^31 bytes. (The first version computed a 64-bit address and a
// row comparison per element: 13 vector instructions, among them a 64-bit multiplication, for every store, 11 us per
// 256 x 256 tile, a sixth of the FP4 kernel's time. What is left, 6-7 us per tile, is the write path itself: 256 KiB
// per compute unit, all compute units at once. Two wider forms were measured and dropped: with the accumulators
// transposed (B as the instruction's first operand) a lane holds four consecutive columns and stores 16 bytes, but a
// store then covers 32 rows x 32 bytes instead of two whole 128-byte lines and the tile took 36 us; with the tiles
// turned through LDS so that a lane stores 16 bytes of a whole row (64 store instructions per wave instead of 256)
// it took the same 7 us as this form.)
template <int FM, int FN, int SCALE_LOG2 = 0, bool ALPHA = false>
__device__ __forceinline__ void store_c_tiles(const f32x16 (&acc)[FM][FN], float* __restrict__ Cb, int64_t M,
                                              int64_t N, int64_t ldc, int64_t row_base, int64_t col_base,
                                              float alpha = 1.0f) {
  const int64_t rows_left = M - row_base, cols_left = N - col_base;  // uniform over the wave
  if (rows_left <= 0 || cols_left <= 0) return;
  const int rows_valid = rows_left < FM * 32 ? (int)rows_left : FM * 32;
  const int cols_valid = cols_left < FN * 32 ? (int)cols_left : FN * 32;
  const uint32_t pitch = (uint32_t)ldc * 4u;
  const __amdgpu_buffer_rsrc_t window = __builtin_amdgcn_make_buffer_rsrc(
      Cb + row_base * ldc + col_base, 0, (int)((uint32_t)(rows_valid - 1) * pitch + (uint32_t)cols_valid * 4u), 0x00020000);
  // the lane number is taken from the hardware again here rather than kept alive (or spilled) across the main loop
  const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int col = j * 32 + (lane & 31);
    const uint32_t lane_off = col < cols_valid ? (uint32_t)col * 4u + (uint32_t)(4 * (lane >> 5)) * pitch : 0x80000000u;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float c = acc[i][j][v];
        if constexpr (SCALE_LOG2 != 0) c *= (float)(1 << SCALE_LOG2);
        if constexpr (ALPHA) c *= alpha;
        const uint32_t row_off = (uint32_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * pitch;
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, c), window, (int)lane_off, (int)row_off,
                                              2 /* non-temporal */);
      }
    }
  }
}

// The gated-activation epilogue: the wave's column tiles come in pairs (gate columns, up columns: the B operand's rows
// are interleaved in blocks of 32), and out[row][c] = bf16(silu(gate) * up) for the 32 columns c of each pair, the
// arithmetic of the separate operator (layer_math.h). out is row-major BF16 with leading dimension ld and n_out
// columns; col_base is the first (interleaved) column of the wave's tiles, a multiple of 64.
// A lane holds single elements of 16 rows per tile, which would make 2-byte stores; the wave therefore transposes its
// result through `stage`, LDS of its own of at least glu_stage_bytes<FM, FN>() bytes (the operand stages, free once
// every wave of the workgroup is past its last fragment read), and stores 16 bytes per lane, whole rows of the
// wave's columns at a time. Needs out 16-byte aligned and ld % 8 == 0; otherwise (and for the columns of a partial
// last chunk) it stores element by element.
template <int FM, int FN>
constexpr int glu_stage_bytes() {
  return FM * 32 * ((FN / 2) * 64 + 16);
}

template <int FM, int FN>
__device__ __forceinline__ void store_glu_tiles(const f32x16 (&acc)[FM][FN], uint8_t* stage, uint16_t* __restrict__ out,
                                                int64_t M, int64_t n_out, int64_t ld, int64_t row_base,
                                                int64_t col_base) {
  static_assert(FN % 2 == 0, "column tiles come in (gate, up) pairs");
  constexpr int kCols = (FN / 2) * 32, kPitch = kCols * 2 + 16;  // bytes per staged row (padded against bank conflicts)
  const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int64_t col0 = col_base >> 1;
  const bool wide = (reinterpret_cast<uintptr_t>(out) & 15) == 0 && (ld & 7) == 0 && col0 + kCols <= n_out;
  if (!wide) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int64_t row0 = row_base + i * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = row0 + 8 * (v >> 2) + (v & 3);
        if (row < M) {
#pragma unroll
          for (int j = 0; j < FN; j += 2) {
            const int64_t col = col0 + (j >> 1) * 32 + (lane & 31);
            if (col < n_out) out[row * ld + col] = (uint16_t)bf16_rne(silu_mul_value(acc[i][j][v], acc[i][j + 1][v]));
          }
        }
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
      for (int j = 0; j < FN; j += 2)
        *reinterpret_cast<uint16_t*>(stage + r * kPitch + ((j >> 1) * 32 + (lane & 31)) * 2) =
            (uint16_t)bf16_rne(silu_mul_value(acc[i][j][v], acc[i][j + 1][v]));
    }
  // (LDS executes a wave's accesses in order: the reads below see the writes above)
  constexpr int kChunks = kCols / 8;            // 16-byte chunks per row
  constexpr int kRowsPerPass = 64 / kChunks;    // rows one store instruction covers
  const int chunk = lane % kChunks, rsub = lane / kChunks;
#pragma unroll
  for (int r0 = 0; r0 < FM * 32; r0 += kRowsPerPass) {
    const int r = r0 + rsub;
    const int64_t row = row_base + r;
    const uint4 val = *reinterpret_cast<const uint4*>(stage + r * kPitch + chunk * 16);
    if (row < M) *reinterpret_cast<uint4*>(out + row * ld + col0 + chunk * 8) = val;
  }
}

}  // namespace amx
