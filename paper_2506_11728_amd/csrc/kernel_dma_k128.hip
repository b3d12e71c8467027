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

namespace mip {

namespace {

constexpr int DM = 256, DN = 256;  // workgroup tile

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
  // Workgroups of the first round (the first first_round workgroup numbers: one per compute
  // unit) start late by their row in the XCD's patch of tiles times stagger_ticks (10 ns
  // each); 0 = all at once.
  int first_round, stagger_ticks;
};

// ---------------------------------------------------------------------------
// 256 x 256 tile, k blocks of 128, two LDS stages for A and three for B: half as many barriers per unit
// of work as the 64-deep kernel, and every row of a k-contiguous operand is fetched as one full
// 128-byte line.  A block is four sub-blocks of 32; the barrier that publishes
// block t+1 sits before the last sub-block of block t, whose fragments are
// already in registers, so the refill of the stage just read starts there.
// ---------------------------------------------------------------------------
constexpr int KD2 = 128;
constexpr int A_STAGE_BYTES = DM * KD2;                // 32 KiB
constexpr int B_STAGE_BYTES = DN * KD2;                // 32 KiB
constexpr int A_STAGES = 2;
// The B blocks have a third stage (160 KB of LDS in all): the loads of B for block t+2 go out
// a whole block earlier than a second stage would allow, and the barrier of step t lets them
// fly on.  What must have landed at a barrier was then issued at least one block of matrix
// instructions before it (with two stages each, the B half had three quarters of a block
// less, too little for a miss in L2).
constexpr int B_STAGES = 3;
constexpr int B_BASE = A_STAGES * A_STAGE_BYTES;
constexpr int LDS2_BYTES = B_BASE + B_STAGES * B_STAGE_BYTES;  // 160 KiB
constexpr int LOADS2 = DM * KD2 / 16 / NTHREADS;       // 8 per operand per thread per block
constexpr int STAGGER_TICKS = 100;                     // 1 us between the rows of an XCD's patch

// UNS: 0 both operands signed, 1 A unsigned, 2 B unsigned.
template <bool A_KC, bool B_KC, int UNS, bool RAGGED = false>
__global__ __launch_bounds__(NTHREADS) void dma128_kernel(DmaParams P) {
  using SA = Stage<DM, A_KC, KD2>;
  using SB = Stage<DN, B_KC, KD2>;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  int tm, tn;
  if (!tile_of_workgroup(P.tiles_m, P.tiles_n, &tm, &tn)) return;
  const int64_t m0 = (int64_t)tm * DM, n0 = (int64_t)tn * DN;
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

  uint32_t offA[LOADS2], offB[LOADS2];
#pragma unroll
  for (int i = 0; i < LOADS2; ++i) {
    int a, c;
    SA::chunk_of(i, tid, a, c);
    offA[i] = A_KC ? (uint32_t)(a * P.lda + ((c ^ SA::kswz(a)) << 4))
                   : (uint32_t)(a * P.lda + ((c ^ SA::swz(a)) << 4));
    SB::chunk_of(i, tid, a, c);
    offB[i] = B_KC ? (uint32_t)(a * P.ldb + ((c ^ SB::kswz(a)) << 4))
                   : (uint32_t)(a * P.ldb + ((c ^ SB::swz(a)) << 4));
  }
  const uint8_t *gA = P.A + (A_KC ? m0 * P.lda : m0);
  const uint8_t *gB = P.B + (B_KC ? n0 * P.ldb : n0);
  const int64_t stepA = A_KC ? KD2 : KD2 * P.lda;
  const int64_t stepB = B_KC ? KD2 : KD2 * P.ldb;

  const uint32_t lds0 = lds_address(smem) + wave * 1024;
  // direct load q (0..7) of the next A block / the next B block into the given stage
  auto issue_a = [&](int stage, int q) { dma16(offA[q], gA, lds0 + stage * A_STAGE_BYTES + q * 4096); };
  auto issue_b = [&](int stage, int q) {
    dma16(offB[q], gB, lds0 + B_BASE + stage * B_STAGE_BYTES + q * 4096);
  };

  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  int sumA[4] = {0, 0, 0, 0}, sumB[4] = {0, 0, 0, 0};  // k sums of the signed operand
  v4i fa[2][4], fb[2][4];
  // unsigned operand: bias its bytes to signed, and sum the other operand over k
  auto prepare = [&](v4i (&a)[4], v4i (&b)[4]) {
    if (UNS == 1) {
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] ^= (int)0x80808080u;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumB[j] = __builtin_amdgcn_sdot4(b[j][r], 0x01010101, sumB[j], false);
    }
    if (UNS == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] ^= (int)0x80808080u;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumA[i] = __builtin_amdgcn_sdot4(a[i][r], 0x01010101, sumA[i], false);
    }
  };
  // fragment f (0..3 of A, 4..7 of B) of sub-block ks of the block in stages (sa, sb)
  auto read_frag = [&](int sa, int sb, int ks, int f, v4i (&a)[4], v4i (&b)[4]) {
    if (f < 4) a[f] = SA::fragment(smem + sa * A_STAGE_BYTES, wm * 128 + f * 32, ks, lane);
    else b[f - 4] = SB::fragment(smem + B_BASE + sb * B_STAGE_BYTES, wn * 128 + (f - 4) * 32, ks, lane);
  };

  const int nkt = P.nkt;  // k / 128
  // prologue: block 0 whole, published; then A and B of block 1 (B of block 2 follows in step 0)
#pragma unroll
  for (int q = 0; q < LOADS2; ++q) issue_a(0, q);
#pragma unroll
  for (int q = 0; q < LOADS2; ++q) issue_b(0, q);
  gA += stepA;
  gB += stepB;
  publish_barrier<0>();
#pragma unroll
  for (int f = 0; f < 8; ++f) read_frag(0, 0, 0, f, fa[0], fb[0]);
  if (nkt > 1) {
#pragma unroll
    for (int q = 0; q < LOADS2; ++q) issue_a(1, q);
#pragma unroll
    for (int q = 0; q < LOADS2; ++q) issue_b(1, q);
    gA += stepA;
    gB += stepB;
  }

  // 16 MFMAs of one sub-block, with up to 8 fragment reads and 8 direct loads between them
  auto phase = [&](int set, auto reader, auto loader) {
    prepare(fa[set], fb[set]);
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      acc[s >> 2][s & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
          fb[set][s & 3], fa[set][s >> 2], acc[s >> 2][s & 3], 0, 0, 0);
      if (s < 8) reader(s);
      else loader(s - 8);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto nothing = [](int) {};

  // Step t multiplies block t (A in stage t % 2, B in stage t % 3 = bcur).  On entry A and B
  // of block t+1 are on their way.  NEXT: block t+1 exists.  NEXT2: block t+2 exists.
  int bcur = 0;
  auto step = [&](int t, auto next_tag, auto next2_tag) {
    constexpr bool NEXT = decltype(next_tag)::value;
    constexpr bool NEXT2 = decltype(next2_tag)::value;
    const int cur = t & 1, oth = cur ^ 1;
    const int bnext = bcur == B_STAGES - 1 ? 0 : bcur + 1;
    const int bfill = bnext == B_STAGES - 1 ? 0 : bnext + 1;  // held block t-1: free since the last barrier
    // sub-block 0; fetch sub-block 1; B of block t+2
    phase(0, [&](int f) { read_frag(cur, bcur, 1, f, fa[1], fb[1]); },
          [&](int q) { if (NEXT2) issue_b(bfill, q); });
    if (NEXT2) gB += stepB;
    phase(1, [&](int f) { read_frag(cur, bcur, 2, f, fa[0], fb[0]); }, nothing);
    phase(0, [&](int f) { read_frag(cur, bcur, 3, f, fa[1], fb[1]); }, nothing);
    // block t+1 visible (only the B loads of block t+2 may still fly); the A stage of block t
    // may be refilled
    if (NEXT) {
      if (NEXT2) publish_barrier<LOADS2>();
      else publish_barrier<0>();
    }
    phase(1, [&](int f) { if (NEXT) read_frag(oth, bnext, 0, f, fa[0], fb[0]); },
          [&](int q) { if (NEXT2) issue_a(cur, q); });
    if (NEXT2) gA += stepA;
    bcur = bnext;
  };
  using std::integral_constant;
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
  // the last step has no barrier of its own: wait until no wave reads the stages any more
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  unsigned_correction<4, 4>(acc, sumA, sumB, UNS == 1, UNS == 2, lane);
  const int64_t mw = m0 + wm * 128, nw = n0 + wn * 128;  // the wave's 128 x 128 patch
  if (P.out_float == 2) {  // int8 output: C is a matrix of bytes
    int8_t *Q = reinterpret_cast<int8_t *>(P.C) + mw * P.ldc + nw;
    if (!RAGGED || (mw + 128 <= P.m && nw + 128 <= P.n))
      store_blocks_q8_via_lds<4, 4>(acc, Q, P.ldc, lane, smem + wave * STORE_PATCH_BYTES, P.scale);
    else if (mw < P.m && nw < P.n)
      store_blocks_q8<4, 4>(acc, Q, P.ldc, P.m - mw, P.n - nw, lane, P.scale);
    return;
  }
  if (!RAGGED || (mw + 128 <= P.m && nw + 128 <= P.n))
    store_blocks_via_lds<4, 4>(acc, P.C + mw * P.ldc + nw, P.ldc, P.accumulate != 0, lane,
                               reinterpret_cast<int32_t *>(smem + wave * STORE_PATCH_BYTES),
                               Finish{P.scale, P.out_float});
  else if (mw < P.m && nw < P.n)
    store_blocks<4, 4, false>(acc, P.C + mw * P.ldc + nw, P.ldc, P.m - mw, P.n - nw,
                              P.accumulate != 0, lane, Finish{P.scale, P.out_float});
}

}  // namespace

bool dma_k128_eligible(const Problem &p) {
  if (p.conv || p.batch != 1 || p.k % KD2 || p.k < KD2) return false;
  // ragged m or n: only on k-contiguous operands padded to whole tiles of rows
  if ((p.m % DM || p.n % DN) && !(p.rows_padded_to_256 && p.a_sk == 1 && p.b_sk == 1)) return false;
  const int64_t lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  const int64_t ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  if (lda % 16 || ldb % 16) return false;
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  if (256 * lda >= ((int64_t)1 << 31) || 256 * ldb >= ((int64_t)1 << 31)) return false;
  if (((p.m + DM - 1) / DM) * ((p.n + DN - 1) / DN) > ((int64_t)1 << 30)) return false;
  return true;
}

hipError_t launch_dma_k128(const Problem &p, hipStream_t s, unsigned long long *clocks) {
  DmaParams P;
  P.clocks = clocks;
  P.A = static_cast<const uint8_t *>(p.A);
  P.B = static_cast<const uint8_t *>(p.B);
  P.C = p.C;
  P.lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  P.ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  P.ldc = p.ldc;
  P.m = p.m;
  P.n = p.n;
  P.tiles_m = (int)((p.m + DM - 1) / DM);
  P.tiles_n = (int)((p.n + DN - 1) / DN);
  P.nkt = (int)(p.k / KD2);
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  const int ntiles = P.tiles_m * P.tiles_n;
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8));
  // (measured at 8192^3, four rounds: 326 -> 310 us on constant operands, 452 -> 444 us on
  // random ones; the 7 us of late start are not earned back by a single round)
  P.first_round = (int)compute_units();
  P.stagger_ticks = ntiles >= 2 * P.first_round ? STAGGER_TICKS : 0;
  const size_t lds = (size_t)LDS2_BYTES;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  const int uns = p.a_unsigned ? 1 : (p.b_unsigned ? 2 : 0);
  void (*kern)(DmaParams) = nullptr;
#define MIP_PICK(AK, BKC)                                                        \
  kern = uns == 0 ? dma128_kernel<AK, BKC, 0>                                    \
                  : (uns == 1 ? dma128_kernel<AK, BKC, 1> : dma128_kernel<AK, BKC, 2>)
  if (p.m % DM || p.n % DN)
    kern = uns == 0 ? dma128_kernel<true, true, 0, true>
                    : (uns == 1 ? dma128_kernel<true, true, 1, true> : dma128_kernel<true, true, 2, true>);
  else if (a_kc && b_kc) MIP_PICK(true, true);
  else if (a_kc) MIP_PICK(true, false);
  else if (b_kc) MIP_PICK(false, true);
  else MIP_PICK(false, false);
#undef MIP_PICK
  hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds, s, P);
  return hipGetLastError();
}

}  // namespace mip
