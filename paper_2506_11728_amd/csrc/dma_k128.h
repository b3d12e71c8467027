#pragma once
// The kernel for large, aligned problems (the m = n = k = 8192 class):
// 256 x 256 tile of C per workgroup, operands streamed global -> LDS directly.
// See dma_tile.h for the general form; this one trades generality for a deeper
// k block.
//
// Preconditions, checked on the host (dma_k128_eligible): m and n multiples of
// 256, k a multiple of 128, 16-byte aligned operand bases and leading
// dimensions, 256 * ld below 2^31.  RAGGED form: any m and n, on k-contiguous
// operands whose buffers are readable up to the next multiple of 256 rows (the
// packed operands of the library's own packing step); whole tiles are loaded and
// multiplied, the write-back stops at the edge of C.
#include "dma_common.h"
#include "epilogue16.h"
#include "tuning.h"

namespace mip {

namespace {

constexpr int DM = 256, DN = 256;  // workgroup tile of the kernel for large problems (a 128 x 128 form serves mid-size ones)

struct DmaParams {
  const uint8_t *A, *B;
  int32_t *C;
  int64_t lda, ldb, ldc;  // the one stride of each operand that is not 1
  int64_t m, n;           // rows and columns of C (RAGGED form only)
  int tiles_m, tiles_n;
  int nkt;                // k / 128
  int accumulate;         // C += instead of C =
  int out_float;          // 1 dequantised output: float(sum) * scale; 2 requantised int8 output
  float scale;
  // not null: workgroup w adds the shader clocks and the 10 ns ticks it ran for to
  // clocks[2 w], clocks[2 w + 1] (benchmarks: the clock the device sustained)
  unsigned long long *clocks;
  // UNS 3 and 4: the k sums of the signed operand, one per column of B (3) or row of A (4)
  const int32_t *ksum;
  // Workgroups of the first round (the first first_round workgroup numbers: one per compute
  // unit) start late by their row in the XCD's patch of tiles times stagger_ticks (10 ns
  // each); 0 = all at once.
  int first_round, stagger_ticks;
  // GENERAL form: k is cut into `splits` ranges of whole blocks, one per blockIdx.y; with
  // `atomic` set the partial sums are added into C with integer atomics (C zeroed or holding
  // the values to add to beforehand).
  int splits, atomic;
};

// ---------------------------------------------------------------------------
// 256 x 256 tile, k blocks of 128, two LDS stages for A and three for B (160 KB), one wave
// per SIMD, each on a 128 x 128 sub-tile held as 8 x 8 blocks of v_mfma_i32_16x16x64_i8.
//
// Why the 16 x 16 x 64 form and not 32 x 32 x 32, which needs half as many instructions:
// the device is power-limited on operands with random bits, and with everything in registers
// the 16 x 16 x 64 form sustains about a fifth more operations per second on such operands
// (it reads and writes a quarter of the accumulator registers per multiply-accumulate); the
// LDS traffic is the same, since that depends on the wave's sub-tile only.
//
// The matrix instructions are written as inline assembly with the accumulators bound to
// the accumulation registers: left to the register allocator, 64 four-register accumulators
// plus two sets of sixteen fragments end up shuffled between the two register files inside
// the loop.  The compiler therefore does not see them as matrix instructions and inserts no
// wait states for them: the kernel never reads an accumulator before the loop has ended and
// two s_nop 15 have passed, and consecutive matrix instructions never share an accumulator.
//
// A k block is two sub-blocks of 64; the barrier that publishes block t+1 sits between the
// two sub-blocks of block t (the fragments of the second are in registers by then), so the A
// stage just read is refilled from there on, while B, with its third stage, is fetched a
// whole block earlier.  A wave issues at most one instruction every four clocks and a matrix
// instruction occupies the pipe for sixteen, so what goes between two matrix instructions
// has to stay within three instructions: the direct loads are spread one per four matrix
// instructions over the first half of a sub-block, the fragment reads one per two over the
// second half, and M0 is set by one scalar add placed before the matrix instruction, which
// then also is the wait state the load needs.
// ---------------------------------------------------------------------------
constexpr int KD2 = 128;
constexpr int A_STAGES = 2;
constexpr int B_STAGES = 3;
constexpr int STAGGER_TICKS = 100;                     // 1 us between the rows of an XCD's patch
constexpr int FIX_LAG = 3;  // fragment reads between a read and its fix-up (unsigned operands)

// Sizes and instruction slots of one tile shape (BM x BN, the four waves 2 x 2 over it).
template <int BM, int BN>
struct Tile16 {
  static constexpr int FM = BM / 32, FN = BN / 32;       // 16 x 16 blocks of a wave's sub-tile
  static constexpr int NMFMA = FM * FN;                   // matrix instructions per sub-block of 64
  static constexpr int NREADS = FM + FN;                  // fragment reads per sub-block
  static constexpr int A_STAGE_BYTES = BM * KD2, B_STAGE_BYTES = BN * KD2;
  static constexpr int B_BASE = A_STAGES * A_STAGE_BYTES;
  static constexpr int LDS_BYTES = B_BASE + B_STAGES * B_STAGE_BYTES;  // 256 x 256: 160 KiB
  static constexpr int LOADS_A = BM * KD2 / 16 / NTHREADS, LOADS_B = BN * KD2 / 16 / NTHREADS;  // per thread and block
  static constexpr int LOADS_MAX = LOADS_A > LOADS_B ? LOADS_A : LOADS_B;
  // matrix instructions per direct load, from the first of a sub-block on (256 x 256: 4)
  static constexpr int LOAD_EVERY = NMFMA / (2 * LOADS_MAX) > 0 ? NMFMA / (2 * LOADS_MAX) : 1;
  // first matrix instruction of a sub-block that is followed by a fragment read, and their spacing
  static constexpr int READ_EVERY = NMFMA >= 64 ? 2 : 1;
  static constexpr int READ_FROM = NMFMA >= 64 ? 24 : NMFMA - (NREADS + FIX_LAG) - 1;
  static_assert(LOAD_EVERY * LOADS_MAX <= NMFMA && READ_FROM >= 0 &&
                READ_FROM + (NREADS + FIX_LAG) * READ_EVERY <= NMFMA, "slots of one sub-block");
};

// One R x 128 operand block in LDS (R = 256 or 128), laid out for the 16 x 16 x 64 instruction.
//   KC (k contiguous in memory): R rows of 128 bytes; 16-byte chunk c of row r sits at
//     r*128 + 16*(c ^ kswz(r)).
//   strided (the index runs contiguously): 128 k-rows of R bytes; chunk c of k-row q sits
//     at q*R + 16*(c ^ swz(q)).
// kswz spreads the sixteen rows one ds_read_b128 group touches over all banks; swz does the
// same for the eight k-rows of one transposing read and, with its lowest bit, lets the lane
// groups that read k-rows 16 apart take the other half of the banks.
template <int R, bool KC>
struct Stage16 {
  static constexpr int ROW_CHUNKS = R / 16;  // strided: chunks per k-row
  __device__ static __forceinline__ int kswz(int r) { return (r >> 1) & 7; }
  // (k-rows 256 bytes apart share banks: R = 256 every row, R = 128 every other one)
  __device__ static __forceinline__ int swz(int q) { return (2 * ((q / (256 / R)) % (R / 32))) ^ ((q >> 4) & 1); }
  // chunk handled by this thread in direct load i: (row, chunk) for KC, (k-row, chunk) otherwise
  __device__ static __forceinline__ void chunk_of(int i, int tid, int &a, int &c) {
    const int q = tid + NTHREADS * i;
    if (KC) { a = q >> 3; c = q & 7; } else { a = q / ROW_CHUNKS; c = q % ROW_CHUNKS; }
  }
  __device__ static __forceinline__ uint32_t global_offset(int i, int tid, int64_t ld) {
    int a, c;
    chunk_of(i, tid, a, c);
    return (uint32_t)(a * ld + ((c ^ (KC ? kswz(a) : swz(a))) << 4));
  }
  // The same for a tile that reaches past the operand's edge: `extent` rows (KC) or bytes of
  // every k-row (strided; a multiple of 16) exist from the tile's origin on.  Chunks beyond
  // that are fetched from a place that does exist; what they feed never reaches C.
  __device__ static __forceinline__ uint32_t global_offset_within(int i, int tid, int64_t ld, int extent) {
    int a, c;
    chunk_of(i, tid, a, c);
    int g = c ^ (KC ? kswz(a) : swz(a));
    if (KC) a = a < extent ? a : extent - 1;
    else g = 16 * g < extent ? g : 0;
    return (uint32_t)(a * ld + (g << 4));
  }
  // The part of a fragment's LDS address that depends on the lane and on the fragment's first
  // row (a multiple of 16); sub-block, stage and, for the transposing reads, the second half
  // of the fragment are constant offsets from it.
  __device__ static __forceinline__ int lane_base(int row0, int lane) {
    if (KC) return (row0 + (lane & 15)) * 128;
    const int s = lane & 15;
    const int col = row0 + (s & 1) * 8;
    const int q = (lane >> 4) * 16 + (s >> 1);
    return q * R + (((col >> 4) ^ swz(q)) << 4) + (col & 15);
  }
  // Fragment for one operand of the instruction: lane l gets, for row (row0 + l % 16), the 16
  // bytes k = 64*ks + 16*(l / 16) .. + 15 of the staged block.
  __device__ static __forceinline__ v4i fragment(const uint8_t *stage, int base, int ks, int lane) {
    if (KC) {
      const int c = ks * 4 + (lane >> 4);
      return *reinterpret_cast<const v4i *>(stage + base + ((c ^ kswz(lane & 15)) << 4));
    }
    // ds_read_b64_tr_b8: inside each group of 16 lanes, lane 2t+h supplies the address of
    // half h of the 16 bytes of k-row t, and lane i receives byte i of k-rows 0..7
    v4i f;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      v2i h = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, stage + base + ks * (64 * R) + t * (8 * R)));
      f[2 * t] = h[0];
      f[2 * t + 1] = h[1];
    }
    return f;
  }
};

// UNS: 0 both operands signed, 1 A unsigned, 2 B unsigned; 3 and 4: as 1 and 2 with the k sums
// of the signed operand read from P.ksum (pre-packed weights carry them) instead of being
// accumulated from the fragments in the loop, which costs four dot-product instructions per
// fragment of the signed operand between the matrix instructions.
//
// GENERAL (with RAGGED): m and n need not be whole tiles and the operands need no padding
// (loads that would leave an operand are redirected inside it); a strided operand's extent
// must be a multiple of 16.  On 128 x 128 tiles k may also be cut into ranges whose partial
// sums meet in C through atomics: the form for problems with too few tiles to occupy the
// device and a long k.
template <int BM, int BN, bool A_KC, bool B_KC, int UNS, bool RAGGED = false, bool GENERAL = false>
__global__ __launch_bounds__(NTHREADS) void dma128_kernel(DmaParams P) {
  constexpr bool FLIP_A = UNS == 1 || UNS == 3, FLIP_B = UNS == 2 || UNS == 4;
  constexpr bool SUM_A = UNS == 2, SUM_B = UNS == 1;
  using TS = Tile16<BM, BN>;
  using SA = Stage16<BM, A_KC>;
  using SB = Stage16<BN, B_KC>;
  constexpr int FM = TS::FM, FN = TS::FN, NMFMA = TS::NMFMA, NREADS = TS::NREADS;
  constexpr int A_STAGE_BYTES = TS::A_STAGE_BYTES, B_STAGE_BYTES = TS::B_STAGE_BYTES, B_BASE = TS::B_BASE;
  constexpr int LOADS_A = TS::LOADS_A, LOADS_B = TS::LOADS_B, LOADS_MAX = TS::LOADS_MAX;
  constexpr int WM = BM / 2, WN = BN / 2;  // a wave's sub-tile
  using std::integral_constant;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  int tm, tn;
  if (!tile_of_workgroup(P.tiles_m, P.tiles_n, &tm, &tn)) return;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  // With several rounds of tiles all compute units would reach their write-backs at the
  // same moments, round after round, and the 32 of one XCD share one path to memory: a tile's
  // stores take about 7 us then, against 3.5 us when only four compute units of an XCD store
  // at a time.  The eight tile rows of an XCD's patch therefore start 1 us apart and stay
  // apart in every later round (the workgroups of one row share their A panel and keep
  // step; a B panel's users drift by a few k blocks, which the L2 still covers).
  if (P.stagger_ticks > 0 && (int)blockIdx.x < P.first_round) {
    const unsigned long long until =
        wall_clock64() + (unsigned long long)((blockIdx.x / 8) % 8) * P.stagger_ticks;
    while (wall_clock64() < until) __builtin_amdgcn_s_sleep(8);
  }
  unsigned long long clock0 = 0, tick0 = 0;
  if (P.clocks) {
    clock0 = __builtin_readcyclecounter();
    tick0 = wall_clock64();
  }

  uint32_t offA[LOADS_MAX], offB[LOADS_MAX];  // (entries past an operand's own count stay unused)
#pragma unroll
  for (int i = 0; i < LOADS_MAX; ++i) {
    if (GENERAL) {
      const int rows_a = (int)(P.m - m0 < BM ? P.m - m0 : BM), rows_b = (int)(P.n - n0 < BN ? P.n - n0 : BN);
      offA[i] = i < LOADS_A ? SA::global_offset_within(i, tid, P.lda, rows_a) : 0;
      offB[i] = i < LOADS_B ? SB::global_offset_within(i, tid, P.ldb, rows_b) : 0;
    } else {
      offA[i] = i < LOADS_A ? SA::global_offset(i, tid, P.lda) : 0;
      offB[i] = i < LOADS_B ? SB::global_offset(i, tid, P.ldb) : 0;
    }
  }
  const int64_t stepA = A_KC ? KD2 : KD2 * P.lda;
  const int64_t stepB = B_KC ? KD2 : KD2 * P.ldb;
  // this workgroup's k blocks: all of them, or range blockIdx.y of P.splits
  const int block0 = GENERAL ? (int)((int64_t)blockIdx.y * P.nkt / P.splits) : 0;
  const int nkt = GENERAL ? (int)((int64_t)(blockIdx.y + 1) * P.nkt / P.splits) - block0 : P.nkt;  // k / 128
  const uint8_t *gA = P.A + (A_KC ? m0 * P.lda : m0) + block0 * stepA;
  const uint8_t *gB = P.B + (B_KC ? n0 * P.ldb : n0) + block0 * stepB;

  const uint32_t lds0 = lds_address(smem) + wave * 1024;
  // direct load q (0..7) of an A block / a B block into the given stage (prologue only: in
  // the loop the loads ride with the matrix instructions)
  auto issue_a = [&](int stage, int q) { dma16(offA[q], gA, lds0 + stage * A_STAGE_BYTES + q * 4096); };
  auto issue_b = [&](int stage, int q) {
    dma16(offB[q], gB, lds0 + B_BASE + stage * B_STAGE_BYTES + q * 4096);
  };

  v4i acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) acc[i][j] = v4i{0, 0, 0, 0};

  int sumA[FM], sumB[FN];  // k sums of the signed operand
  v4i fa[2][FM], fb[2][FN];
  int baseA[FM], baseB[FN];
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    sumA[f] = 0;
    baseA[f] = SA::lane_base(wm * WM + f * 16, lane);
  }
#pragma unroll
  for (int f = 0; f < FN; ++f) {
    sumB[f] = 0;
    baseB[f] = SB::lane_base(wn * WN + f * 16, lane);
  }
  // read r of a sub-block's FN + FM fragments, B's first: the first row of matrix
  // instructions needs all of B's and one of A's
  auto read_frag = [&](int sa, int sb, int ks, int r, v4i (&a)[FM], v4i (&b)[FN]) {
    if (r < FN) b[r] = SB::fragment(smem + B_BASE + sb * B_STAGE_BYTES, baseB[r], ks, lane);
    else a[r - FN] = SA::fragment(smem + sa * A_STAGE_BYTES, baseA[r - FN], ks, lane);
  };
  // Unsigned operand: bias its bytes to signed and sum the other operand over k.  Done to
  // fragment r of a set a few matrix instructions after its read was issued and well before
  // the sub-block that uses the set begins: the matrix instructions are inline assembly, so
  // nothing inserts the wait states they need after an ordinary instruction has written
  // one of their operands.
  auto fix_frag = [&](int r, v4i (&a)[FM], v4i (&b)[FN]) {
    if (r < FN) {
      if (FLIP_B) b[r] ^= (int)0x80808080u;
      if (SUM_B) {
#pragma unroll
        for (int e = 0; e < 4; ++e) sumB[r] = __builtin_amdgcn_sdot4(b[r][e], 0x01010101, sumB[r], false);
      }
    } else {
      if (FLIP_A) a[r - FN] ^= (int)0x80808080u;
      if (SUM_A) {
#pragma unroll
        for (int e = 0; e < 4; ++e) sumA[r - FN] = __builtin_amdgcn_sdot4(a[r - FN][e], 0x01010101, sumA[r - FN], false);
      }
    }
  };
  // Supplied k sums: the lane that would hold the first quarter of a row's (column's) sum takes
  // the whole of it, the other three lane groups zero, and the correction below adds them up
  // as it does the accumulated ones.  Read here, ahead of the loop, which hides the latency.
  if (UNS == 3) {
#pragma unroll
    for (int f = 0; f < FN; ++f) {
      const int64_t col = n0 + wn * WN + f * 16 + (lane & 15);
      sumB[f] = lane < 16 && (!RAGGED || col < P.n) ? P.ksum[col] : 0;
    }
  }
  if (UNS == 4) {
#pragma unroll
    for (int f = 0; f < FM; ++f) {
      const int64_t row = m0 + wm * WM + f * 16 + (lane & 15);
      sumA[f] = lane < 16 && (!RAGGED || row < P.m) ? P.ksum[row] : 0;
    }
  }
  // prologue: block 0 whole, published; then A and B of block 1 (B of block 2 follows in step 0)
#pragma unroll
  for (int q = 0; q < LOADS_A; ++q) issue_a(0, q);
#pragma unroll
  for (int q = 0; q < LOADS_B; ++q) issue_b(0, q);
  gA += stepA;
  gB += stepB;
  publish_barrier<0>();
#pragma unroll
  for (int r = 0; r < NREADS; ++r) read_frag(0, 0, 0, r, fa[0], fb[0]);
  if (UNS != 0) {
#pragma unroll
    for (int r = 0; r < NREADS; ++r) fix_frag(r, fa[0], fb[0]);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 7" ::: "memory");  // k = 128: nothing else before the first matrix instruction
    __builtin_amdgcn_sched_barrier(0);
  }
  if (nkt > 1) {
#pragma unroll
    for (int q = 0; q < LOADS_A; ++q) issue_a(1, q);
#pragma unroll
    for (int q = 0; q < LOADS_B; ++q) issue_b(1, q);
    gA += stepA;
    gB += stepB;
  }

  // The FM x FN matrix instructions of one sub-block on fragment set `set`, row by row of the
  // blocks, odd rows backwards so that only one operand changes from one instruction to the
  // next.  LOADS > 0: that many of them carry one direct load each, into the stage at LDS
  // address `ldsbase` from gbase + off[q].
  auto phase = [&](int set, auto reader, auto fixer, auto loads_tag, uint32_t ldsbase,
                   const uint32_t (&off)[LOADS_MAX], const uint8_t *gbase) {
    constexpr int LOADS = decltype(loads_tag)::value;
    constexpr int LOAD_EVERY = TS::LOAD_EVERY, READ_FROM = TS::READ_FROM, READ_EVERY = TS::READ_EVERY;
#pragma unroll
    for (int s = 0; s < NMFMA; ++s) {
      const int i = s / FN, j = (i & 1) ? FN - 1 - (s % FN) : (s % FN);
      if (s % LOAD_EVERY == 0 && s / LOAD_EVERY < LOADS) {
        asm volatile(
            "s_add_u32 m0, %3, %4\n\t"
            "v_mfma_i32_16x16x64_i8 %0, %1, %2, %0\n\t"
            "global_load_lds_dwordx4 %5, %6"
            : "+a"(acc[i][j])
            : "v"(fb[set][j]), "v"(fa[set][i]), "s"(ldsbase), "i"((s / LOAD_EVERY) * 4096),
              "v"(off[s / LOAD_EVERY]), "s"(gbase)
            : "scc");
      } else {
        asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0"
                     : "+a"(acc[i][j])
                     : "v"(fb[set][j]), "v"(fa[set][i]));
      }
      if (s >= READ_FROM && (s - READ_FROM) % READ_EVERY == 0) {
        const int r = (s - READ_FROM) / READ_EVERY;
        if (r < NREADS) reader(r);
        if (UNS != 0 && r >= FIX_LAG && r - FIX_LAG < NREADS) fixer(r - FIX_LAG);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Step t multiplies block t (A in stage t % 2, B in stage t % 3 = bcur).  On entry A and B
  // of block t+1 are on their way.  NEXT: block t+1 exists.  NEXT2: block t+2 exists.
  int bcur = 0;
  auto step = [&](int t, auto next_tag, auto next2_tag) {
    constexpr bool NEXT = decltype(next_tag)::value;
    constexpr bool NEXT2 = decltype(next2_tag)::value;
    const int cur = t & 1, oth = cur ^ 1;
    const int bnext = bcur == B_STAGES - 1 ? 0 : bcur + 1;
    const int bfill = bnext == B_STAGES - 1 ? 0 : bnext + 1;  // held block t-1: free since the last barrier
    // first sub-block; fetch the second; B of block t+2
    phase(0, [&](int r) { read_frag(cur, bcur, 1, r, fa[1], fb[1]); },
          [&](int r) { fix_frag(r, fa[1], fb[1]); }, integral_constant<int, NEXT2 ? LOADS_B : 0>{},
          lds0 + B_BASE + bfill * B_STAGE_BYTES, offB, gB);
    if (NEXT2) gB += stepB;
    // block t+1 visible (only the B loads of block t+2 may still fly); the A stage of block t
    // may be refilled
    if (NEXT) {
      if (NEXT2) publish_barrier<LOADS_B>();
      else publish_barrier<0>();
    }
    phase(1, [&](int r) { if (NEXT) read_frag(oth, bnext, 0, r, fa[0], fb[0]); },
          [&](int r) { if (NEXT) fix_frag(r, fa[0], fb[0]); }, integral_constant<int, NEXT2 ? LOADS_A : 0>{},
          lds0 + cur * A_STAGE_BYTES, offA, gA);
    if (NEXT2) gA += stepA;
    bcur = bnext;
  };
  using T = integral_constant<bool, true>;
  using F = integral_constant<bool, false>;
  int t = 0;
  for (; t + 2 < nkt; ++t) step(t, T{}, T{});
  if (t + 1 < nkt) { step(t, T{}, F{}); ++t; }
  step(t, F{}, F{});

  if (P.clocks && tid == 0) {  // the main loop alone: what the matrix pipe saw
    P.clocks[2 * blockIdx.x] += __builtin_readcyclecounter() - clock0;
    P.clocks[2 * blockIdx.x + 1] += wall_clock64() - tick0;
  }
  // The last matrix instructions have to leave the pipe before an accumulator is read (the
  // compiler does not know that the statements above write them late); the last step has no
  // barrier of its own: wait until no wave reads the stages any more.
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  int32_t *patch = reinterpret_cast<int32_t *>(smem) + wave * Patch16<FN>::WORDS;
  // (the corrections of an unsigned operand: behind the four patches, one area per wave)
  const Correction16<FM, FN> corr = unsigned_correction16<FM, FN>(
      sumA, sumB, FLIP_A, FLIP_B, lane,
      reinterpret_cast<int32_t *>(smem) + 4 * Patch16<FN>::WORDS + wave * Correction16<FM, FN>::WORDS);
  const int64_t mw = m0 + wm * WM, nw = n0 + wn * WN;  // the wave's sub-tile
  // an int8 output is a matrix of bytes, ldc counted in bytes
  void *C = P.out_float == 2 ? static_cast<void *>(reinterpret_cast<int8_t *>(P.C) + mw * P.ldc + nw)
                             : static_cast<void *>(P.C + mw * P.ldc + nw);
  bool added = false;
  if constexpr (GENERAL && BM == 128 && BN == 128) {  // (k ranges exist on the small tile only)
    if (P.atomic) {
      if (mw < P.m && nw < P.n)
        add_blocks16_atomic<FM, FN, UNS != 0>(acc, P.C + mw * P.ldc + nw, P.ldc, P.m - mw, P.n - nw, lane, patch, corr);
      added = true;
    }
  }
  if (added) {
  } else if (!RAGGED || (mw + WM <= P.m && nw + WN <= P.n))
    store_blocks16<FM, FN, true, UNS != 0>(acc, C, P.ldc, WM, WN, P.accumulate != 0, P.out_float, lane, patch,
                                           P.scale, corr);
  else if (mw < P.m && nw < P.n)
    store_blocks16<FM, FN, false, UNS != 0>(acc, C, P.ldc, P.m - mw, P.n - nw, P.accumulate != 0, P.out_float,
                                            lane, patch, P.scale, corr);
}

}  // namespace

}  // namespace mip
