// Write-back of the register-resident accumulator blocks (the paper's C_r,
// Section 4.1: loaded or zeroed before loop L6, stored once after it), shared
// by the MFMA kernels.
//
// The kernels issue v_mfma_i32_32x32x32_i8 with the B fragment as first operand
// and the A fragment as second, so each 32 x 32 block comes out transposed in
// the register file: lane l owns C row (l % 32) of the block and register v
// owns column 8*(v/4) + 4*(l/32) + v%4.  Four consecutive registers are four
// consecutive int32 of one row of C: one 16-byte store per lane.
#pragma once
#include "lds_layout.h"

namespace mip {

struct __attribute__((packed, aligned(4))) c_quad { v4i v; };

// What becomes of an accumulator on its way to C.  Integer output: the sum
// itself, plus the old C when accumulating (wraps modulo 2^32).  Dequantised
// output (paper Section 7.3, C^r = s_A s_B C^q): the int32 sum converted to
// float (round to nearest even) times `scale`; when accumulating, one fused
// multiply-add onto the old float.  Both views of C are 4-byte words, so the
// stores below move bit patterns.
struct Finish {
  float scale;
  int to_float;  // 0 int32, 1 float; 2 = requantised int8 output, which has write-back loops of its own
  __device__ __forceinline__ int operator()(int acc, int old, bool accumulate) const {
    if (!to_float) return accumulate ? (int)((uint32_t)acc + (uint32_t)old) : acc;
    const float s = (float)acc;
    const float r = accumulate ? __fmaf_rn(s, scale, __int_as_float(old)) : __fmul_rn(s, scale);
    return __float_as_int(r);
  }
};
typedef v4i v4i_dword_aligned __attribute__((aligned(4)));  // four int32 of C: only dword alignment is known

// The same with the case fixed at compile time: MODE bit 0 = accumulate (the old word is
// needed), bit 1 = float output.  The write-back loops are instantiated once per MODE and
// entered through a wave-uniform switch: a loop that has to allow for the old words of C
// carries waits on the memory counter between its stores, and that counter counts stores as
// well, so an overwriting call written that way keeps only a handful of stores in flight per
// wave (measured on 256 x 256 tiles: 10 us to issue a tile's 64 stores per lane, the same
// whether one compute unit stores or all of them).  The overwriting instances have no loads
// and therefore no such waits.
template <int MODE>
struct FinishAs {
  float scale;
  static constexpr bool ACCUMULATE = (MODE & 1) != 0;
  static constexpr bool TO_FLOAT = (MODE & 2) != 0;
  __device__ __forceinline__ int operator()(int acc, int old) const {
    if (!TO_FLOAT) return ACCUMULATE ? (int)((uint32_t)acc + (uint32_t)old) : acc;
    const float s = (float)acc;
    const float r = ACCUMULATE ? __fmaf_rn(s, scale, __int_as_float(old)) : __fmul_rn(s, scale);
    return __float_as_int(r);
  }
};
__device__ __forceinline__ int finish_mode(const Finish &fin, bool accumulate) {
  return (accumulate ? 1 : 0) | (fin.to_float ? 2 : 0);
}

// Unsigned-operand correction (exact modulo 2^32).  sumB[j]: this lane's partial
// sum over k of column (32*j + l%32) of the staged B; sumA[i]: same for row
// (32*i + l%32) of A; lanes l and l^32 hold the two k halves.
template <int FM, int FN>
__device__ __forceinline__ void unsigned_correction(v16i (&acc)[FM][FN], const int (&sumA)[FM],
                                                    const int (&sumB)[FN], bool a_unsigned,
                                                    bool b_unsigned, int lane) {
  if (a_unsigned) {  // sum_p (a - 128) b + 128 sum_p b: needs B's column sums
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int total = sumB[j] + __shfl_xor(sumB[j], 32);  // lane l: column l % 32
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int col = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int corr = 128 * __shfl(total, col);
#pragma unroll
        for (int i = 0; i < FM; ++i) acc[i][j][v] += corr;
      }
    }
  }
  if (b_unsigned) {  // needs A's row sums, which already sit in the owning lane
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int corr = 128 * (sumA[i] + __shfl_xor(sumA[i], 32));
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += corr;
    }
  }
}

// C points at the first element of the wave's sub-tile; rows / cols are how
// many of its 32*FM x 32*FN elements lie inside the matrix.
template <int FM, int FN, bool FULL, int MODE>
__device__ __forceinline__ void store_blocks_as(const v16i (&acc)[FM][FN], int32_t *C, int64_t ldc,
                                                int64_t rows, int64_t cols, int lane,
                                                const FinishAs<MODE> fin) {
  constexpr bool ACCUMULATE = FinishAs<MODE>::ACCUMULATE;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int row = i * 32 + (lane & 31);
    if (!FULL && row >= rows) continue;
    int32_t *crow = C + row * ldc + 4 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      // an accumulating call has the old words of all four pieces of the block in flight
      // before the first store (a load behind every store would wait for it in turn)
      v4i old[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
      bool whole[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = j * 32 + 8 * q;  // plus 4 * (lane / 32), already in crow
        whole[q] = FULL || col + 4 * (lane >> 5) + 3 < cols;
        if (ACCUMULATE && whole[q]) old[q] = reinterpret_cast<const c_quad *>(crow + col)->v;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = j * 32 + 8 * q;
        v4i val = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                   acc[i][j][4 * q + 3]};
        if (whole[q]) {
#pragma unroll
          for (int e = 0; e < 4; ++e) val[e] = fin(val[e], old[q][e]);
          reinterpret_cast<c_quad *>(crow + col)->v = val;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (col + 4 * (lane >> 5) + e < cols)
              crow[col + e] = fin(val[e], ACCUMULATE ? crow[col + e] : 0);
          }
        }
      }
    }
  }
}

template <int FM, int FN, bool FULL>
__device__ __forceinline__ void store_blocks(const v16i (&acc)[FM][FN], int32_t *C, int64_t ldc,
                                             int64_t rows, int64_t cols, bool accumulate,
                                             int lane, const Finish fin) {
  switch (finish_mode(fin, accumulate)) {  // wave-uniform
    case 0: store_blocks_as<FM, FN, FULL, 0>(acc, C, ldc, rows, cols, lane, FinishAs<0>{fin.scale}); break;
    case 1: store_blocks_as<FM, FN, FULL, 1>(acc, C, ldc, rows, cols, lane, FinishAs<1>{fin.scale}); break;
    case 2: store_blocks_as<FM, FN, FULL, 2>(acc, C, ldc, rows, cols, lane, FinishAs<2>{fin.scale}); break;
    default: store_blocks_as<FM, FN, FULL, 3>(acc, C, ldc, rows, cols, lane, FinishAs<3>{fin.scale}); break;
  }
}

// Write-back of full tiles through a wave-private patch of LDS.  Straight from
// registers, one store instruction covers 32 bytes of each of 32 rows of C, so
// every 128-byte line of C is completed by four separate instructions; turned
// through LDS, one instruction writes 8 whole lines.  The stores are marked
// non-temporal: C is written once and never read by this kernel, and letting it
// allocate in L2 evicts the operand panels the other workgroups are streaming.
// Measured on the 8192^3 case: 4 % faster on random operands, 20 % on constant
// ones, against direct cached stores.
// `patch` is this wave's STORE_PATCH_BYTES of LDS; the caller has made sure that
// no wave still reads operand stages from LDS.
constexpr int STORE_PATCH_WORDS = 32 * 36;
constexpr int STORE_PATCH_BYTES = STORE_PATCH_WORDS * 4;

// An accumulating call reads the old words of C up to three 32 x 32 blocks ahead of the block
// it is writing, so that their latency hides behind the turns through LDS and the stores of
// the blocks before (loaded only when needed, a store per load in turn, the 2048^3 case took
// 25.1 us against 15.5 us for an overwriting call; one block ahead 18.7 us).
// STREAM: the stores are non-temporal.  That pays when the row pieces are whole cache lines; rows
// of C that start at odd words leave every line to be completed by a neighbouring piece, which
// only a store that stays in L2 until then can be merged with.
template <int FM, int FN, int MODE, bool STREAM>
__device__ __forceinline__ void store_blocks_via_lds_as(const v16i (&acc)[FM][FN], int32_t *C,
                                                        int64_t ldc, int lane, int32_t *patch,
                                                        const FinishAs<MODE> fin) {
  constexpr bool ACCUMULATE = FinishAs<MODE>::ACCUMULATE;
  constexpr int NB = FM * FN;
  constexpr int AHEAD = ACCUMULATE ? (NB < 3 ? NB : 3) : 1;  // blocks of old words in registers
  // the piece of a 32 x 32 block this lane handles in pass t: 4 words of row t * 8 + lane / 8
  const int r0 = lane >> 3, c0 = (lane & 7) * 4;
  auto piece = [&](int block, int t) {
    const int i = block / FN, j = block % FN;
    return reinterpret_cast<v4i_dword_aligned *>(C + (int64_t)(i * 32 + t * 8 + r0) * ldc + j * 32 + c0);
  };
  v4i old[AHEAD][4];
#pragma unroll
  for (int b = 0; b < AHEAD; ++b)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      old[b][t] = v4i{0, 0, 0, 0};
      if (ACCUMULATE) old[b][t] = STREAM ? __builtin_nontemporal_load(piece(b, t)) : *piece(b, t);
    }
#pragma unroll
  for (int block = 0; block < NB; ++block) {
    const int i = block / FN, j = block % FN;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v4i val = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                 acc[i][j][4 * q + 3]};
      *reinterpret_cast<v4i *>(patch + (lane & 31) * 36 + 8 * q + 4 * (lane >> 5)) = val;
    }
    // same wave wrote and reads: LDS operations of a wave complete in order
    v4i val[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
      val[t] = *reinterpret_cast<const v4i *>(patch + (t * 8 + r0) * 36 + c0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int e = 0; e < 4; ++e) val[t][e] = fin(val[t][e], old[block % AHEAD][t][e]);
      if (STREAM) __builtin_nontemporal_store(val[t], piece(block, t));
      else *piece(block, t) = val[t];
    }
    if (ACCUMULATE && block + AHEAD < NB) {  // the slot just used takes the block AHEAD further on
#pragma unroll
      for (int t = 0; t < 4; ++t)
        old[block % AHEAD][t] = STREAM ? __builtin_nontemporal_load(piece(block + AHEAD, t)) : *piece(block + AHEAD, t);
    }
  }
}

template <int FM, int FN>
__device__ __forceinline__ void store_blocks_via_lds(const v16i (&acc)[FM][FN], int32_t *C,
                                                     int64_t ldc, bool accumulate, int lane,
                                                     int32_t *patch, const Finish fin) {
  // whole 128-byte lines per row piece: rows start on a line and are a whole number of lines apart
  const bool lines = reinterpret_cast<uintptr_t>(C) % 128 == 0 && ldc % 32 == 0;
  switch (finish_mode(fin, accumulate) + (lines ? 0 : 4)) {  // wave-uniform
    case 0: store_blocks_via_lds_as<FM, FN, 0, true>(acc, C, ldc, lane, patch, FinishAs<0>{fin.scale}); break;
    case 1: store_blocks_via_lds_as<FM, FN, 1, true>(acc, C, ldc, lane, patch, FinishAs<1>{fin.scale}); break;
    case 2: store_blocks_via_lds_as<FM, FN, 2, true>(acc, C, ldc, lane, patch, FinishAs<2>{fin.scale}); break;
    case 3: store_blocks_via_lds_as<FM, FN, 3, true>(acc, C, ldc, lane, patch, FinishAs<3>{fin.scale}); break;
    case 4: store_blocks_via_lds_as<FM, FN, 0, false>(acc, C, ldc, lane, patch, FinishAs<0>{fin.scale}); break;
    case 5: store_blocks_via_lds_as<FM, FN, 1, false>(acc, C, ldc, lane, patch, FinishAs<1>{fin.scale}); break;
    case 6: store_blocks_via_lds_as<FM, FN, 2, false>(acc, C, ldc, lane, patch, FinishAs<2>{fin.scale}); break;
    default: store_blocks_via_lds_as<FM, FN, 3, false>(acc, C, ldc, lane, patch, FinishAs<3>{fin.scale}); break;
  }
}

// Split-k write-back: every workgroup adds its partial sums into C with integer
// atomics (order-independent, so still bit-exact).  The blocks sit transposed in
// registers (lane = row), which would scatter one atomic instruction over 64
// cache lines; each block is turned through a wave-private 32 x 33 word patch of
// LDS so that the lanes of one instruction cover 32 consecutive columns of a row.
// `patch` is this wave's 4224-byte LDS area; the caller has made sure that no
// wave still reads operand stages from LDS.
constexpr int ATOMIC_PATCH_BYTES = 32 * 33 * 4;

template <int FM, int FN>
__device__ __forceinline__ void add_blocks_atomic(const v16i (&acc)[FM][FN], int32_t *C,
                                                  int64_t ldc, int64_t rows, int64_t cols,
                                                  int lane, int32_t *patch) {
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      if (i * 32 >= rows || j * 32 >= cols) continue;  // wave-uniform
#pragma unroll
      for (int v = 0; v < 16; ++v)
        patch[(lane & 31) * 33 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] = acc[i][j][v];
      // same wave wrote and reads: LDS operations of a wave complete in order
      const int col = j * 32 + (lane & 31);
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int r = 2 * t + (lane >> 5);
        const int val = patch[r * 33 + (lane & 31)];
        const int row = i * 32 + r;
        if (row < rows && col < cols) atomicAdd(C + row * ldc + col, val);
      }
    }
  }
}

// Requantised output (paper Section 7.3, X ~ s_X X^q, applied to the product: the int32 sum
// brought into the int8 scale of the next layer): Q = clip(rint(scale * S), -128, 127), the
// sum converted to float (nearest even), one float multiplication, rounding to the nearest
// integer with ties to even, saturation.  C is a matrix of BYTES here (ldc counts bytes).
__device__ __forceinline__ int requantise(int sum, float scale) {
  float r = __builtin_rintf(__fmul_rn((float)sum, scale));
  r = fminf(fmaxf(r, -128.0f), 127.0f);
  return (int)r & 0xff;
}

struct __attribute__((packed, aligned(1))) q8_run { v4i v; };  // 16 output bytes at any address

// The blocks sit transposed in the registers (lane = row of C, four consecutive registers =
// four consecutive columns): four sums make one packed word, and a lane and its partner 32
// lanes on, which hold alternate words of the same row, swap two words each so that every
// lane ends up with 16 consecutive bytes of its row.  One 16-byte store per lane and block;
// at a ragged edge the bytes go out one by one.
template <int FM, int FN>
__device__ __forceinline__ void store_blocks_q8(const v16i (&acc)[FM][FN], int8_t *C, int64_t ldc,
                                                int64_t rows, int64_t cols, int lane, float scale) {
  const int h = lane >> 5;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int row = i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      int word[4];  // word q: columns 8 q + 4 h .. + 3 of the block
#pragma unroll
      for (int q = 0; q < 4; ++q)
        word[q] = requantise(acc[i][j][4 * q], scale) | requantise(acc[i][j][4 * q + 1], scale) << 8 |
                  requantise(acc[i][j][4 * q + 2], scale) << 16 |
                  requantise(acc[i][j][4 * q + 3], scale) << 24;
      // the lower half of the wave keeps columns 0..15 (its words 0, 1 and the partner's),
      // the upper half columns 16..31
      const int got0 = __shfl_xor(h ? word[0] : word[2], 32);
      const int got1 = __shfl_xor(h ? word[1] : word[3], 32);
      const v4i run = h ? v4i{got0, word[2], got1, word[3]} : v4i{word[0], got0, word[1], got1};
      const int col = j * 32 + 16 * h;
      if (row >= rows || col >= cols) continue;
      int8_t *dst = C + row * ldc + col;
      if (col + 16 <= cols) {
        reinterpret_cast<q8_run *>(dst)->v = run;
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (col + e < cols) dst[e] = (int8_t)(run[e >> 2] >> (8 * (e & 3)));
      }
    }
  }
}

// The same for a sub-tile that lies wholly inside the matrix, turned through the wave's LDS
// patch so that one store instruction writes whole rows of the sub-tile, 32 * FN bytes each
// (FN = 4: eight full 128-byte lines per instruction, where the direct form above leaves 32
// bytes in each of 32 lines).  `patch` is this wave's STORE_PATCH_BYTES of LDS; the caller
// has made sure that no wave still reads operand stages from LDS.
template <int FM, int FN>
__device__ __forceinline__ void store_blocks_q8_via_lds(const v16i (&acc)[FM][FN], int8_t *C,
                                                        int64_t ldc, int lane, uint8_t *patch,
                                                        float scale) {
  static_assert(FN >= 2 && FN <= 4, "rows of 64 to 128 bytes");
  constexpr int PITCH = 32 * FN + 16;          // bytes; 32 rows fit the patch for FN <= 4
  constexpr int LANES_PER_ROW = 2 * FN;        // 16 bytes each
  constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
  const int h = lane >> 5, r = lane & 31;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      int word[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        word[q] = requantise(acc[i][j][4 * q], scale) | requantise(acc[i][j][4 * q + 1], scale) << 8 |
                  requantise(acc[i][j][4 * q + 2], scale) << 16 |
                  requantise(acc[i][j][4 * q + 3], scale) << 24;
      const int got0 = __shfl_xor(h ? word[0] : word[2], 32);
      const int got1 = __shfl_xor(h ? word[1] : word[3], 32);
      const v4i run = h ? v4i{got0, word[2], got1, word[3]} : v4i{word[0], got0, word[1], got1};
      *reinterpret_cast<v4i *>(patch + r * PITCH + j * 32 + 16 * h) = run;
    }
    // same wave wrote and reads: LDS operations of a wave complete in order
#pragma unroll
    for (int t = 0; t < 32 / ROWS_PER_PASS; ++t) {
      const int row = t * ROWS_PER_PASS + lane / LANES_PER_ROW, piece = lane % LANES_PER_ROW;
      const v4i v = *reinterpret_cast<const v4i *>(patch + row * PITCH + piece * 16);
      reinterpret_cast<q8_run *>(C + (int64_t)(i * 32 + row) * ldc + piece * 16)->v = v;
    }
  }
}

// Split k without atomics and without a zeroed C: every workgroup of a tile writes its partial
// sums into its own slot of a caller-supplied buffer (register order: one coalesced 16-byte
// store per lane), then takes a ticket; the workgroup that draws the last ticket adds the
// other slots to its own registers and goes on to the ordinary write-back, so that any mode
// and a float output work as in an unsplit call (the sum is complete, in integers, before
// anything is converted).  Nobody waits for anybody.  `slots` points at the tile's `splits`
// slots of 4 * FM * FN * 1024 words; `ticket` at the tile's counter, which is zero on entry
// and zero again when the last workgroup leaves.  Returns true in the workgroup that holds
// the complete sums.  Integer addition is associative: the result is the same bits whichever
// workgroup comes last.
//
// Visibility between workgroups, which may run on different XCDs with L2 caches of their
// own: every slot access carries the device-scope bit (sc1: the store is written through to
// the level all XCDs share, the load is served from there), a workgroup draws its ticket, a
// device-scope atomic, only after its stores have been acknowledged (vmcnt 0), and the last
// workgroup issues its loads only after its ticket has come back.  Device-wide fences, which
// write back and invalidate a whole L2, are not needed and were measured to cost about
// 0.1 us per workgroup serialised per XCD (2048^3 in 2 x 2048 workgroups: 350 us).
__device__ __forceinline__ void store16_device_scope(v4i *p, v4i v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ v4i load16_device_scope(const v4i *p) {
  v4i v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
  return v;  // in flight: the caller waits with loads_landed before touching it
}
// "the loads issued above have landed": ties the registers to the wait, so that nothing that
// uses them is scheduled before it
__device__ __forceinline__ void loads_landed(v4i &a, v4i &b, v4i &c, v4i &d) {
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)::"memory");
}

template <int FM, int FN>
__device__ __forceinline__ bool combine_k_ranges(v16i (&acc)[FM][FN], int32_t *slots, int range,
                                                 int splits, unsigned *ticket, int wave, int lane,
                                                 int tid, int *lds_word) {
  constexpr int WAVE_WORDS = FM * FN * 1024;
  constexpr int SLOT_WORDS = 4 * WAVE_WORDS;
  v4i *mine = reinterpret_cast<v4i *>(slots + (int64_t)range * SLOT_WORDS + wave * WAVE_WORDS) + lane;
#pragma unroll
  for (int b = 0; b < FM * FN; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      store16_device_scope(mine + (b * 4 + q) * 64,
                           v4i{acc[b / FN][b % FN][4 * q], acc[b / FN][b % FN][4 * q + 1],
                               acc[b / FN][b % FN][4 * q + 2], acc[b / FN][b % FN][4 * q + 3]});
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the slot has arrived where every XCD reads it
  __syncthreads();
  if (tid == 0) *lds_word = atomicAdd(ticket, 1u) == (unsigned)(splits - 1) ? 1 : 0;
  __syncthreads();
  if (!*lds_word) return false;
  for (int r = 0; r < splits; ++r) {
    if (r == range) continue;
    const v4i *other =
        reinterpret_cast<const v4i *>(slots + (int64_t)r * SLOT_WORDS + wave * WAVE_WORDS) + lane;
#pragma unroll
    for (int b = 0; b < FM * FN; ++b) {
      v4i v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = load16_device_scope(other + (b * 4 + q) * 64);
      loads_landed(v[0], v[1], v[2], v[3]);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[b / FN][b % FN][4 * q + e] = (int)((uint32_t)acc[b / FN][b % FN][4 * q + e] + (uint32_t)v[q][e]);
    }
  }
  if (tid == 0) atomicExch(ticket, 0u);  // every range has drawn: the counter is free again
  return true;
}

}  // namespace mip
