// The large-problem kernel: 256 x 256 tile of C per workgroup, operands streamed
// global -> LDS without passing through registers (global_load_lds_dwordx4),
// four LDS stages, one workgroup barrier per 64-deep k block.
//
// In the paper's terms (Section 3 and Section 4.1): the 256 x 64 block of A and
// the 64 x 256 block of B that a workgroup holds in LDS are the packed buffers
// A_c and B_c; "packing" is done by the choice of which 16-byte piece each lane
// fetches, so that the piece lands where the fragment reads expect it.  The
// micro-kernel is v_mfma_i32_32x32x32_i8 on a 128 x 128 register-resident
// accumulator block per wave (C_r), stored once after the k loop.
//
// Preconditions, checked on the host (dma_eligible): m and n multiples of 256,
// k a multiple of 64, 16-byte aligned operand bases and leading dimensions,
// 256 * ld below 2^31.  Everything else takes the generic tile kernel.
#include <type_traits>

#include "epilogue.h"
#include "lds_layout.h"
#include "mip_internal.h"

namespace mip {

namespace {

constexpr int DM = 256, DN = 256;        // workgroup tile
constexpr int STAGES = 4;
constexpr int STAGE_BYTES = (DM + DN) * BK;  // 32 KiB
constexpr int LOADS = DM * BK / 16 / NTHREADS;  // 16-byte pieces per thread, per operand, per k block

struct DmaParams {
  const uint8_t *A, *B;
  int32_t *C;
  int64_t lda, ldb, ldc;  // the one stride of each operand that is not 1
  int tiles_m, tiles_n;
  int nkt;                // k / 64
};

// One wave-wide direct load: lane l's 16 bytes from sbase + voff land in LDS at
// lds_addr + 16 * l.  Written as inline assembly so that the compiler's
// automatic wait-count insertion, which would drain every outstanding load
// before any LDS read, stays out of the pipeline; the kernel places its own
// s_waitcnt vmcnt before the barrier that publishes a stage.  M0 carries the
// LDS base and needs one wait state before the load reads it.
__device__ __forceinline__ void dma16(uint32_t voff, const uint8_t *sbase, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(sbase), "s"(lds_addr)
      :);  // M0 is reserved: the compiler keeps nothing live in it across statements
}

// "my loads of the next block have landed (N newer loads may still fly), my LDS
// reads are complete; meet the other waves": after this the next stage is
// visible to the whole workgroup and the stage read two steps ago may be refilled.
template <int N>
__device__ __forceinline__ void publish_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const uint8_t *p) {
  return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const uint8_t *)p);
}

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHREADS) void dma_kernel(DmaParams P) {
  using SA = Stage<DM, A_KC>;
  using SB = Stage<DN, B_KC>;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // workgroup -> tile: contiguous run of tiles per XCD, tiles walked in groups of 8 tile-rows
  const int ntiles = P.tiles_m * P.tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  const int lid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (lid >= ntiles) return;
  constexpr int GROUP = 8;
  const int per_group = GROUP * P.tiles_n;
  const int first_m = (lid / per_group) * GROUP;
  const int gsz = P.tiles_m - first_m < GROUP ? P.tiles_m - first_m : GROUP;
  const int tm = first_m + (lid % per_group) % gsz;
  const int tn = (lid % per_group) / gsz;
  const int64_t m0 = (int64_t)tm * DM, n0 = (int64_t)tn * DN;

  // Per-lane source offsets.  LDS piece Q = i*256 + tid of an operand block holds the
  // logical piece whose swizzled position is Q (the XOR is its own inverse).
  uint32_t offA[LOADS], offB[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
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
  const int64_t stepA = A_KC ? BK : BK * P.lda;
  const int64_t stepB = B_KC ? BK : BK * P.ldb;

  const uint32_t lds0 = lds_address(smem) + wave * 1024;
  // one of the 8 direct loads of a k block (0..3: A, 4..7: B)
  auto issue_one = [&](int stage, int q) {
    const uint32_t sa = lds0 + stage * STAGE_BYTES;
    if (q < LOADS) dma16(offA[q], gA, sa + q * 4096);
    else dma16(offB[q - LOADS], gB, sa + DM * BK + (q - LOADS) * 4096);
  };
  auto advance = [&]() {
    gA += stepA;
    gB += stepB;
  };
  auto issue = [&](int stage) {
#pragma unroll
    for (int q = 0; q < 2 * LOADS; ++q) issue_one(stage, q);
    advance();
  };

  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  const int nkt = P.nkt;
  // prologue: blocks 0 .. STAGES-2 in flight
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nkt) issue(s);

  v4i fa[2][4], fb[2][4];
  // fragment f of a k sub-block: 0..3 rows of A, 4..7 columns of B
  auto read_frag = [&](int stage, int ks, int f, v4i (&a)[4], v4i (&b)[4]) {
    const uint8_t *sa = smem + stage * STAGE_BYTES;
    if (f < 4) a[f] = SA::fragment(sa, wm * 128 + f * 32, ks, lane);
    else b[f - 4] = SB::fragment(sa + DM * BK, wn * 128 + (f - 4) * 32, ks, lane);
  };
  auto read_frags = [&](int stage, int ks, v4i (&a)[4], v4i (&b)[4]) {
#pragma unroll
    for (int f = 0; f < 8; ++f) read_frag(stage, ks, f, a, b);
  };

  constexpr int PER_BLOCK = 2 * LOADS;  // direct loads per thread per k block

  // block 0 visible to everyone, its first fragments on their way
  if (nkt > 2) publish_barrier<2 * PER_BLOCK>();
  else if (nkt > 1) publish_barrier<PER_BLOCK>();
  else publish_barrier<0>();
  read_frags(0, 0, fa[0], fb[0]);

  // One k block of 64 = two sub-blocks of 32, 16 MFMAs each.  The instruction
  // order is pinned (sched_barrier after every slot) so that LDS reads and direct
  // loads sit between MFMAs and their latency hides behind the matrix pipe:
  //   sub-block 0 MFMAs, with the fragment reads of sub-block 1 and, if ISSUE, the
  //                      direct loads of block t+3 (into the stage read in step t-1)
  //   publish barrier    block t+1 becomes visible
  //   sub-block 1 MFMAs, with the fragment reads of block t+1, sub-block 0
  // NEWER: whole blocks that may still be in flight when block t+1 must be
  // complete; -1 marks the last block (nothing to publish).
  auto step = [&](int t, auto issue_tag, auto newer_tag) {
    constexpr bool ISSUE = decltype(issue_tag)::value;
    constexpr int NEWER = decltype(newer_tag)::value;
    const int stage = t & (STAGES - 1);
    const int fill = (t + STAGES - 1) & (STAGES - 1);
    const int next = (t + 1) & (STAGES - 1);
    // Direct loads go out one every other MFMA slot, spread over the whole step:
    // the four waves run in lockstep, and the address unit takes about 16 cycles
    // per wave-wide load, so bunching them stalls the MFMA stream.
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      acc[s >> 2][s & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[0][s & 3], fa[0][s >> 2],
                                                                 acc[s >> 2][s & 3], 0, 0, 0);
      if (s < 8) read_frag(stage, 1, s, fa[1], fb[1]);
      else if (ISSUE && (s & 1)) issue_one(fill, (s - 8) >> 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    // block t+2 and, if issuing, the first half of block t+3 may still be in flight
    if (NEWER >= 0) publish_barrier<ISSUE ? PER_BLOCK + PER_BLOCK / 2 : (NEWER > 0 ? NEWER : 0) * PER_BLOCK>();
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      acc[s >> 2][s & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[1][s & 3], fa[1][s >> 2],
                                                                 acc[s >> 2][s & 3], 0, 0, 0);
      if (NEWER >= 0 && s < 8) read_frag(next, 0, s, fa[0], fb[0]);
      else if (ISSUE && (s & 1)) issue_one(fill, LOADS + ((s - 8) >> 1));
      __builtin_amdgcn_sched_barrier(0);
    }
    if (ISSUE) advance();
  };
  using std::integral_constant;
  int t = 0;
  for (; t + STAGES - 1 < nkt; ++t)  // blocks t+1, t+2, t+3 exist; t+2 and t+3 may fly
    step(t, integral_constant<bool, true>{}, integral_constant<int, 2>{});
  // the last (up to) three blocks: nothing left to issue
  if (t + 2 < nkt) { step(t, integral_constant<bool, false>{}, integral_constant<int, 1>{}); ++t; }
  if (t + 1 < nkt) { step(t, integral_constant<bool, false>{}, integral_constant<int, 0>{}); ++t; }
  step(t, integral_constant<bool, false>{}, integral_constant<int, -1>{});

  // write-back: C_r -> C, one 16-byte store per lane and register quad
  store_blocks<4, 4, true>(acc, P.C + (m0 + wm * 128) * P.ldc + n0 + wn * 128, P.ldc, 128, 128,
                           false, lane);
}


// ---------------------------------------------------------------------------
// Same tile, k blocks of 128 in two LDS stages: half as many barriers per unit
// of work, and every row of a k-contiguous operand is fetched as one full
// 128-byte line.  A block is four sub-blocks of 32; the barrier that publishes
// block t+1 sits before the last sub-block of block t, whose fragments are
// already in registers, so the refill of the stage just read starts there.
// ---------------------------------------------------------------------------
constexpr int KD2 = 128;
constexpr int STAGE2_BYTES = (DM + DN) * KD2;          // 64 KiB
constexpr int LOADS2 = DM * KD2 / 16 / NTHREADS;       // 8 per operand per thread per block

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHREADS) void dma128_kernel(DmaParams P) {
  using SA = Stage<DM, A_KC, KD2>;
  using SB = Stage<DN, B_KC, KD2>;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int ntiles = P.tiles_m * P.tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  const int lid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (lid >= ntiles) return;
  constexpr int GROUP = 8;
  const int per_group = GROUP * P.tiles_n;
  const int first_m = (lid / per_group) * GROUP;
  const int gsz = P.tiles_m - first_m < GROUP ? P.tiles_m - first_m : GROUP;
  const int tm = first_m + (lid % per_group) % gsz;
  const int tn = (lid % per_group) / gsz;
  const int64_t m0 = (int64_t)tm * DM, n0 = (int64_t)tn * DN;

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
  // direct load q of a block: 0..7 A, 8..15 B
  auto issue_one = [&](int stage, int q) {
    const uint32_t sa = lds0 + stage * STAGE2_BYTES;
    if (q < LOADS2) dma16(offA[q], gA, sa + q * 4096);
    else dma16(offB[q - LOADS2], gB, sa + DM * KD2 + (q - LOADS2) * 4096);
  };
  auto advance = [&]() {
    gA += stepA;
    gB += stepB;
  };

  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  v4i fa[2][4], fb[2][4];
  auto read_frag = [&](int stage, int ks, int f, v4i (&a)[4], v4i (&b)[4]) {
    const uint8_t *sa = smem + stage * STAGE2_BYTES;
    if (f < 4) a[f] = SA::fragment(sa, wm * 128 + f * 32, ks, lane);
    else b[f - 4] = SB::fragment(sa + DM * KD2, wn * 128 + (f - 4) * 32, ks, lane);
  };

  const int nkt = P.nkt;  // k / 128
  // prologue: block 0 whole, published; then the first half of block 1
#pragma unroll
  for (int q = 0; q < 2 * LOADS2; ++q) issue_one(0, q);
  advance();
  publish_barrier<0>();
#pragma unroll
  for (int f = 0; f < 8; ++f) read_frag(0, 0, f, fa[0], fb[0]);
  if (nkt > 1) {
#pragma unroll
    for (int q = 0; q < LOADS2; ++q) issue_one(1, q);
  }

  // 16 MFMAs of one sub-block, with up to 8 fragment reads and 8 direct loads between them
  auto phase = [&](int set, auto reader, auto loader) {
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

  // NEXT: block t+1 exists.  NEXT2: block t+2 exists.
  auto step = [&](int t, auto next_tag, auto next2_tag) {
    constexpr bool NEXT = decltype(next_tag)::value;
    constexpr bool NEXT2 = decltype(next2_tag)::value;
    const int cur = t & 1, oth = cur ^ 1;
    // sub-block 0; fetch sub-block 1; second half of block t+1 (first half went out in step t-1)
    phase(0, [&](int f) { read_frag(cur, 1, f, fa[1], fb[1]); },
          [&](int q) { if (NEXT) issue_one(oth, LOADS2 + q); });
    if (NEXT) advance();
    phase(1, [&](int f) { read_frag(cur, 2, f, fa[0], fb[0]); }, nothing);
    phase(0, [&](int f) { read_frag(cur, 3, f, fa[1], fb[1]); }, nothing);
    if (NEXT) publish_barrier<0>();  // block t+1 visible; stage `cur` may be refilled
    phase(1, [&](int f) { if (NEXT) read_frag(oth, 0, f, fa[0], fb[0]); },
          [&](int q) { if (NEXT2) issue_one(cur, q); });
  };
  using std::integral_constant;
  using T = integral_constant<bool, true>;
  using F = integral_constant<bool, false>;
  int t = 0;
  for (; t + 2 < nkt; ++t) step(t, T{}, T{});
  if (t + 1 < nkt) { step(t, T{}, F{}); ++t; }
  step(t, F{}, F{});

  store_blocks<4, 4, true>(acc, P.C + (m0 + wm * 128) * P.ldc + n0 + wn * 128, P.ldc, 128, 128,
                           false, lane);
}

}  // namespace

bool dma_eligible(const Problem &p, bool deep) {
  if (deep && p.k % KD2) return false;
  if (p.a_unsigned || p.b_unsigned || p.accumulate) return false;
  if (p.m % DM || p.n % DN || p.k % BK || p.k < BK) return false;
  const int64_t lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  const int64_t ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  if (lda % 16 || ldb % 16) return false;
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  if (256 * lda >= ((int64_t)1 << 31) || 256 * ldb >= ((int64_t)1 << 31)) return false;
  if ((p.m / DM) * (p.n / DN) > ((int64_t)1 << 30)) return false;
  return true;
}

hipError_t launch_dma(const Problem &p, bool deep, hipStream_t s) {
  DmaParams P;
  P.A = static_cast<const uint8_t *>(p.A);
  P.B = static_cast<const uint8_t *>(p.B);
  P.C = p.C;
  P.lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  P.ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  P.ldc = p.ldc;
  P.tiles_m = (int)(p.m / DM);
  P.tiles_n = (int)(p.n / DN);
  P.nkt = (int)(p.k / (deep ? KD2 : BK));
  const int ntiles = P.tiles_m * P.tiles_n;
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8));
  const size_t lds = deep ? (size_t)2 * STAGE2_BYTES : (size_t)STAGES * STAGE_BYTES;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  void (*kern)(DmaParams) =
      deep ? (a_kc ? (b_kc ? dma128_kernel<true, true> : dma128_kernel<true, false>)
                   : (b_kc ? dma128_kernel<false, true> : dma128_kernel<false, false>))
           : (a_kc ? (b_kc ? dma_kernel<true, true> : dma_kernel<true, false>)
                   : (b_kc ? dma_kernel<false, true> : dma_kernel<false, false>));
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds, s, P);
  return hipGetLastError();
}

}  // namespace mip
