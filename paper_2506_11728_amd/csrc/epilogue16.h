// Write-back of accumulator blocks produced by v_mfma_i32_16x16x64_i8 (the paper's C_r,
// Section 4.1: kept in registers over loop L6, stored once after it).
//
// The kernel issues the instruction with the B fragment as first operand and the A fragment
// as second, so each 16 x 16 block comes out transposed in the register file: lane l owns C
// row (l % 16) of the block and its four registers are columns 4 * (l / 16) .. + 3, four
// consecutive int32 of one row of C.  A wave's sub-tile is FM x FN such blocks.
#pragma once
#include "epilogue.h"

namespace mip {

// Unsigned-operand correction (exact modulo 2^32): what has to be added to every element of
// row r of the wave's sub-tile (rows[r]) and of column c (cols[c]).  Kept in LDS, in an area of
// 16 * (FM + FN) words private to the wave, and added after the blocks have been turned into
// rows of C (one four-word read per lane for its columns, one word per row piece): adding it
// on the way into LDS instead takes every accumulator through the ordinary registers together
// with 5 * FN correction registers, which an accumulating call, with the old words of C in
// flight as well, has no room for.
// sumA[i]: this lane's partial sum over k of row (16 i + l % 16) of the staged A, the four lane
// groups l / 16 holding four quarters of every 64 k; sumB[j]: the same for column
// (16 j + l % 16) of B.
template <int FM, int FN>
struct Correction16 {
  const int32_t *rows;  // 16 * FM words
  const int32_t *cols;  // 16 * FN words
  static constexpr int WORDS = 16 * (FM + FN);
};

// area: Correction16<FM, FN>::WORDS words of LDS that no wave reads as operand stages any more.
template <int FM, int FN>
__device__ __forceinline__ Correction16<FM, FN> unsigned_correction16(const int (&sumA)[FM],
                                                                      const int (&sumB)[FN],
                                                                      bool a_unsigned, bool b_unsigned,
                                                                      int lane, int32_t *area) {
  if (!a_unsigned && !b_unsigned) return Correction16<FM, FN>{area, area + 16 * FM};  // never read
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    int total = 0;
    if (b_unsigned) {  // sum_p a (b - 128) + 128 sum_p a: needs A's row sums
      total = sumA[i] + __shfl_xor(sumA[i], 16);
      total += __shfl_xor(total, 32);  // every lane: row l % 16 of block row i
    }
    if (lane < 16) area[16 * i + lane] = 128 * total;
  }
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    int total = 0;
    if (a_unsigned) {  // sum_p (a - 128) b + 128 sum_p b: needs B's column sums
      total = sumB[j] + __shfl_xor(sumB[j], 16);
      total += __shfl_xor(total, 32);  // every lane: column l % 16 of block column j
    }
    if (lane < 16) area[16 * (FM + j) + lane] = 128 * total;
  }
  return Correction16<FM, FN>{area, area + 16 * FM};
}

// The wave's patch of LDS for the write-back: 16 rows of 16 * FN words, rows 4 words further
// apart than their length so that the sixteen lanes of one access never share a bank.
template <int FN>
struct Patch16 {
  static constexpr int PITCH = 16 * FN + 4;  // words
  static constexpr int WORDS = 16 * PITCH;
  static constexpr int BYTES = 4 * WORDS;
};

struct __attribute__((packed, aligned(1))) q8_word { int w; };  // four output bytes at any address

// Write-back of a wave's sub-tile, sixteen rows at a time turned through the wave's LDS patch
// so that a store instruction covers whole rows of the sub-tile (FN = 8: two rows of 512
// bytes, four full 128-byte lines each; straight from the registers it would leave 64 bytes in
// each of 16 lines).  The stores are non-temporal: C is written once and never read by this
// kernel, and letting it allocate in L2 evicts the operand panels other workgroups stream.
// MODE bit 0: accumulate (the old word is read), bit 1: float output (the dequantised
// product of paper Section 7.3), 4: requantised int8 output, C a matrix of bytes and ldc
// counted in bytes.  FULL: the sub-tile lies wholly inside the matrix; otherwise rows and
// cols say how much of it does, and stores at the edge go out element by element.
// C points at the first element of the sub-tile; `patch` is the wave's Patch16<FN>::WORDS of
// LDS, which no wave still reads as operand stages.
template <int FM, int FN, int MODE, bool FULL, bool CORRECT>
__device__ __forceinline__ void store_blocks16_as(const v4i (&acc)[FM][FN], void *Cv, int64_t ldc,
                                                  int64_t rows, int64_t cols, int lane,
                                                  int32_t *patch, float scale,
                                                  const Correction16<FM, FN> &corr) {
  static_assert(FN == 8 || FN == 4 || FN == 2, "rows of 32 to 128 words");
  constexpr bool Q8 = MODE == 4;
  constexpr bool ACCUMULATE = !Q8 && (MODE & 1);
  constexpr int PITCH = Patch16<FN>::PITCH;
  constexpr int LANES_PER_ROW = 4 * FN;              // four words each
  constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;  // FN = 8: 2
  constexpr int PASSES = 16 / ROWS_PER_PASS;
  const FinishAs<Q8 ? 0 : MODE> fin{scale};
  const int r0 = lane / LANES_PER_ROW, c0 = 4 * (lane % LANES_PER_ROW);
  int32_t *C = static_cast<int32_t *>(Cv);
  int8_t *Q = static_cast<int8_t *>(Cv);
  // An accumulating call reads the old words of a strip of sixteen rows one strip ahead: the
  // loads of strip i + 1 are in flight while strip i is turned and stored, so that only the
  // first strip's load latency is exposed (4096^3 accumulating 79 -> 74 us).
  constexpr bool AHEAD = ACCUMULATE;
  // (same wave wrote the corrections: LDS operations of a wave complete in order)
  const v4i colc = CORRECT ? *reinterpret_cast<const v4i *>(corr.cols + c0) : v4i{0, 0, 0, 0};
  v4i old[2][PASSES];
  auto fetch_old = [&](int i, v4i (&into)[PASSES]) {
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
      const int row = i * 16 + t * ROWS_PER_PASS + r0;
      into[t] = v4i{0, 0, 0, 0};
      if (FULL || (row < rows && c0 + 3 < cols))
        into[t] = __builtin_nontemporal_load(reinterpret_cast<const v4i_dword_aligned *>(C + row * ldc + c0));
    }
  };
  if (AHEAD) fetch_old(0, old[0]);
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    if (!FULL && i * 16 >= rows) break;  // wave-uniform
    if (ACCUMULATE) {
      if (i + 1 < FM) fetch_old(i + 1, old[(i + 1) & 1]);
      // keep the loads up here, in flight during the turn: under register pressure the
      // scheduler otherwise sinks each load to its use and the wave waits for them one by one
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j)
      *reinterpret_cast<v4i *>(patch + (lane & 15) * PITCH + 16 * j + 4 * (lane >> 4)) = acc[i][j];
    // same wave wrote and reads: LDS operations of a wave complete in order
    v4i val[PASSES];
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
      val[t] = *reinterpret_cast<const v4i *>(patch + (t * ROWS_PER_PASS + r0) * PITCH + c0);
      if (CORRECT) val[t] += colc + corr.rows[i * 16 + t * ROWS_PER_PASS + r0];
    }
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
      const int row = i * 16 + t * ROWS_PER_PASS + r0;
      const bool whole = FULL || (row < rows && c0 + 3 < cols);
      if (Q8) {
        const int word = requantise(val[t][0], scale) | requantise(val[t][1], scale) << 8 |
                         requantise(val[t][2], scale) << 16 | requantise(val[t][3], scale) << 24;
        int8_t *dst = Q + row * ldc + c0;
        if (whole) {
          reinterpret_cast<q8_word *>(dst)->w = word;
        } else if (row < rows) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c0 + e < cols) dst[e] = (int8_t)(word >> (8 * e));
        }
      } else {
        int32_t *dst = C + row * ldc + c0;
        if (whole) {
          v4i out;
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = fin(val[t][e], ACCUMULATE ? old[i & 1][t][e] : 0);
          __builtin_nontemporal_store(out, reinterpret_cast<v4i_dword_aligned *>(dst));
        } else if (row < rows) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c0 + e < cols) dst[e] = fin(val[t][e], ACCUMULATE ? dst[e] : 0);
        }
      }
    }
  }
}

// Split k: the wave's partial sums are added into an int32 C with integer atomics (any order
// gives the same bits).  Sixteen rows at a time go through the wave's LDS patch, as in the
// write-back above, so that the 64 lanes of one atomic instruction cover 64 consecutive
// words of one row (two cache lines) instead of four words in each of sixteen rows.
// rows, cols: how much of the sub-tile lies inside the matrix.
template <int FM, int FN, bool CORRECT>
__device__ __forceinline__ void add_blocks16_atomic(const v4i (&acc)[FM][FN], int32_t *C, int64_t ldc,
                                                    int64_t rows, int64_t cols, int lane, int32_t *patch,
                                                    const Correction16<FM, FN> &corr) {
  static_assert(FN == 4, "rows of 64 words: one per lane");
  constexpr int PITCH = Patch16<FN>::PITCH;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    if (i * 16 >= rows) break;  // wave-uniform
#pragma unroll
    for (int j = 0; j < FN; ++j)
      *reinterpret_cast<v4i *>(patch + (lane & 15) * PITCH + 16 * j + 4 * (lane >> 4)) = acc[i][j];
    // same wave wrote and reads: LDS operations of a wave complete in order
    int val[16];
#pragma unroll
    for (int r = 0; r < 16; ++r)
      val[r] = patch[r * PITCH + lane] + (CORRECT ? corr.cols[lane] + corr.rows[i * 16 + r] : 0);
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (i * 16 + r < rows && lane < cols)
        __hip_atomic_fetch_add(C + (i * 16 + r) * ldc + lane, val[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// out_mode: 0 int32, 1 float, 2 int8 (the Problem's out_float).
template <int FM, int FN, bool FULL, bool CORRECT>
__device__ __forceinline__ void store_blocks16(const v4i (&acc)[FM][FN], void *C, int64_t ldc,
                                               int64_t rows, int64_t cols, bool accumulate,
                                               int out_mode, int lane, int32_t *patch, float scale,
                                               const Correction16<FM, FN> &corr) {
  const int mode = out_mode == 2 ? 4 : ((accumulate ? 1 : 0) | (out_mode == 1 ? 2 : 0));
  switch (mode) {  // wave-uniform
    case 0: store_blocks16_as<FM, FN, 0, FULL, CORRECT>(acc, C, ldc, rows, cols, lane, patch, scale, corr); break;
    case 1: store_blocks16_as<FM, FN, 1, FULL, CORRECT>(acc, C, ldc, rows, cols, lane, patch, scale, corr); break;
    case 2: store_blocks16_as<FM, FN, 2, FULL, CORRECT>(acc, C, ldc, rows, cols, lane, patch, scale, corr); break;
    case 3: store_blocks16_as<FM, FN, 3, FULL, CORRECT>(acc, C, ldc, rows, cols, lane, patch, scale, corr); break;
    default: store_blocks16_as<FM, FN, 4, FULL, CORRECT>(acc, C, ldc, rows, cols, lane, patch, scale, corr); break;
  }
}

}  // namespace mip
