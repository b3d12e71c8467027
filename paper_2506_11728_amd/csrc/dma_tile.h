// MFMA tile kernel with operands streamed global -> LDS directly
// (global_load_lds_dwordx4), four LDS stages of 64-deep k blocks and one
// workgroup barrier per block.  Tile shapes from 64 x 64 to 256 x 256, split k,
// unsigned operands, accumulate mode and ragged m / n edges.
//
// In the paper's terms (Section 3 and Section 4.1): the BM x 64 block of A and
// the 64 x BN block of B that a workgroup holds in an LDS stage are the packed
// buffers A_c and B_c; "packing" is the choice of which 16-byte piece each lane
// fetches, so that the piece lands where the fragment reads expect it (storage
// order and leading dimension are absorbed there).  The micro-kernel is
// v_mfma_i32_32x32x32_i8 on the register-resident accumulator blocks of each
// wave (C_r), written back once after the k loop.
//
// Preconditions, checked on the host (dma_tile_eligible): k a multiple of 64;
// operand bases and leading dimensions 16-byte aligned; an operand whose index
// (m or n) runs contiguously in memory needs that extent to be a multiple of
// 16; BM * lda and BN * ldb (or 64 * ld for the strided forms) below 2^31.
// Rows past a ragged edge are fetched from a clamped, valid address and never
// stored.  Everything else takes the register-staged tile kernel.
//
// CONV: A is the lowered matrix of a convolution (paper Section 7.2) that is never
// written out: row i is an output position, and the 64 bytes of a k block are 64
// channels of one filter tap (c_i a multiple of 64), read straight from the image
// tensor; a tap that falls outside the image reads a block of zeros instead.
#pragma once
#include "dma_common.h"

namespace mip {

constexpr int DMA_STAGES = 4;

struct DmaTileParams {
  const uint8_t *A, *B;
  int32_t *C;
  int64_t m, n;
  int64_t lda, ldb, ldc;  // the one stride of each operand that is not 1
  int tiles_m, tiles_n;
  int nkt;                // k / 64 in the whole problem
  int kt_per_split;       // k blocks per workgroup (blockIdx.y picks the range)
  int accumulate;         // C += instead of C =
  int atomic;             // several workgroups add into the same tile (split k)
  // split k through partial-sum slots instead (see combine_k_ranges): `splits` slots per tile
  // in `slots`, one zeroed counter per tile in `tickets`; null = not used
  int32_t *slots;
  unsigned *tickets;
  int splits;
  int out_float;          // 1 dequantised output: float(sum) * scale; 2 requantised int8 output
  float scale;
  const int32_t *ksum;    // UNS 3 and 4: the k sums of the signed operand (see Problem::ksum)
  ConvGeom conv;          // CONV kernels only
  int64_t a_sb, b_sb, c_sb;  // byte / element offsets of problem z of a batch (blockIdx.z)
};

// what a tap outside the image contributes
static __device__ __attribute__((aligned(16))) const uint8_t conv_zero_block[16] = {};

// UNS: 0 both operands signed, 1 A unsigned, 2 B unsigned; 3 and 4: as 1 and 2 with the k sums
// of the signed operand read from P.ksum instead of being accumulated from the fragments
// (whole problem only: with split k every range would add them).
template <int BM, int BN, bool A_KC, bool B_KC, int UNS, bool CONV = false>
__global__ __launch_bounds__(NTHREADS) void dma_tile_kernel(DmaTileParams P) {
  constexpr bool FLIP_A = UNS == 1 || UNS == 3, FLIP_B = UNS == 2 || UNS == 4;
  constexpr bool SUM_A = UNS == 2, SUM_B = UNS == 1;
  static_assert(!CONV || (A_KC && B_KC), "the lowered matrix and the filters are k-contiguous");
  using SA = Stage<BM, A_KC>;
  using SB = Stage<BN, B_KC>;
  constexpr int FM = BM / 64, FN = BN / 64;      // 32 x 32 blocks per wave, down and across
  constexpr int LA = SA::PER_THREAD, LB = SB::PER_THREAD;  // direct loads per thread per block
  constexpr int PER_BLOCK = LA + LB;
  constexpr int STAGE_BYTES = (BM + BN) * BK;
  constexpr int NM = FM * FN;                    // MFMAs per 32-deep sub-block
  constexpr int NF = FM + FN;                    // fragments per sub-block
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  int tm, tn;
  if (!tile_of_workgroup(P.tiles_m, P.tiles_n, &tm, &tn)) return;
  if (!CONV) {  // problem of the batch
    const int64_t z = blockIdx.z;
    P.A += z * P.a_sb;
    P.B += z * P.b_sb;
    P.C += z * P.c_sb;
  }
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int kt_begin = blockIdx.y * P.kt_per_split;
  const int kt_end = kt_begin + P.kt_per_split < P.nkt ? kt_begin + P.kt_per_split : P.nkt;
  const int nkt = kt_end - kt_begin;  // blocks this workgroup works through
  if (nkt <= 0) return;

  // Per-lane source offsets.  LDS piece Q = i*256 + tid of an operand block holds
  // the logical piece whose swizzled position is Q (the XOR is its own inverse).
  // Rows (or 16-wide column groups) past the edge of the matrix are redirected
  // to row (group) 0 of the tile, which always exists.
  const int rows_a = (int)(P.m - m0 < BM ? P.m - m0 : BM);
  const int rows_b = (int)(P.n - n0 < BN ? P.n - n0 : BN);
  uint32_t offA[LA], offB[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    int a, c;
    SA::chunk_of(i, tid, a, c);
    if (A_KC) {
      offA[i] = (uint32_t)((a < rows_a ? a : 0) * P.lda + ((c ^ SA::kswz(a)) << 4));
    } else {
      const int piece = c ^ SA::swz(a);
      offA[i] = (uint32_t)(a * P.lda + ((piece * 16 < rows_a ? piece : 0) << 4));
    }
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    int a, c;
    SB::chunk_of(i, tid, a, c);
    if (B_KC) {
      offB[i] = (uint32_t)((a < rows_b ? a : 0) * P.ldb + ((c ^ SB::kswz(a)) << 4));
    } else {
      const int piece = c ^ SB::swz(a);
      offB[i] = (uint32_t)(a * P.ldb + ((piece * 16 < rows_b ? piece : 0) << 4));
    }
  }
  const int64_t stepA = A_KC ? BK : BK * P.lda;
  const int64_t stepB = B_KC ? BK : BK * P.ldb;
  const uint8_t *gA = P.A + (A_KC ? m0 * P.lda : m0) + kt_begin * stepA;
  const uint8_t *gB = P.B + (B_KC ? n0 * P.ldb : n0) + kt_begin * stepB;

  // CONV: where the window of each of this lane's rows starts in the image (top-left
  // tap; may lie outside), as pixel coordinates and as a byte offset that already
  // includes the lane's 16-byte piece; and the tap / channel block the next loads fetch
  int conv_iy[CONV ? LA : 1], conv_ix[CONV ? LA : 1], conv_at[CONV ? LA : 1];
  int cur_y = 0, cur_x = 0, cur_c = 0, cur_at = 0;
  if constexpr (CONV) {
    const ConvGeom &G = P.conv;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      int a, c;
      SA::chunk_of(i, tid, a, c);
      int64_t row = m0 + a;
      if (row >= P.m) row = P.m - 1;  // past the edge: repeat the last position, never stored
      const int per_image = G.ho * G.wo;
      const int g = (int)(row / per_image), r = (int)(row - (int64_t)g * per_image);
      const int oy = r / G.wo, ox = r - oy * G.wo;
      conv_iy[i] = oy * G.stride - G.pad;
      conv_ix[i] = ox * G.stride - G.pad;
      conv_at[i] = ((g * G.hi + conv_iy[i]) * G.wi + conv_ix[i]) * G.ci + ((c ^ SA::kswz(a)) << 4);
    }
    const int per_tap = G.ci / BK, tap = kt_begin / per_tap;
    cur_c = (kt_begin - tap * per_tap) * BK;
    cur_y = tap / G.wf;
    cur_x = tap - cur_y * G.wf;
    cur_at = (cur_y * G.wi + cur_x) * G.ci + cur_c;
  }

  const uint32_t lds0 = lds_address(smem) + wave * 1024;
  // direct load q of a block: 0 .. LA-1 from A, then LB from B
  auto issue_one = [&](int stage, int q) {
    const uint32_t sa = lds0 + stage * STAGE_BYTES;
    if (q < LA) {
      if constexpr (CONV) {
        const bool inside = (unsigned)(conv_iy[q] + cur_y) < (unsigned)P.conv.hi &&
                            (unsigned)(conv_ix[q] + cur_x) < (unsigned)P.conv.wi;
        dma16_at(inside ? P.A + (conv_at[q] + cur_at) : conv_zero_block, sa + q * 4096);
      } else {
        dma16(offA[q], gA, sa + q * 4096);
      }
    } else {
      dma16(offB[q - LA], gB, sa + BM * BK + (q - LA) * 4096);
    }
  };
  auto advance = [&]() {
    if constexpr (CONV) {
      cur_c += BK;
      if (cur_c == P.conv.ci) {  // next filter tap
        cur_c = 0;
        if (++cur_x == P.conv.wf) {
          cur_x = 0;
          ++cur_y;
        }
      }
      cur_at = (cur_y * P.conv.wi + cur_x) * P.conv.ci + cur_c;
    } else {
      gA += stepA;
    }
    gB += stepB;
  };

  v16i acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
  int sumA[FM], sumB[FN];  // per lane: partial sum over k of its row of A / column of B
#pragma unroll
  for (int i = 0; i < FM; ++i) sumA[i] = 0;
#pragma unroll
  for (int j = 0; j < FN; ++j) sumB[j] = 0;

  // prologue: blocks 0 .. STAGES-2 in flight
#pragma unroll
  for (int s = 0; s < DMA_STAGES - 1; ++s)
    if (s < nkt) {
#pragma unroll
      for (int q = 0; q < PER_BLOCK; ++q) issue_one(s, q);
      advance();
    }

  v4i fa[2][FM], fb[2][FN];
  // fragment f of a k sub-block: 0 .. FM-1 rows of A, then FN columns of B
  auto read_frag = [&](int stage, int ks, int f, v4i (&a)[FM], v4i (&b)[FN]) {
    const uint8_t *sa = smem + stage * STAGE_BYTES;
    if (f < FM) a[f] = SA::fragment(sa, wm * (BM / 2) + f * 32, ks, lane);
    else b[f - FM] = SB::fragment(sa + BM * BK, wn * (BN / 2) + (f - FM) * 32, ks, lane);
  };
  // unsigned operand: bias its bytes to signed, and sum the other operand over k
  auto prepare = [&](v4i (&a)[FM], v4i (&b)[FN]) {
    if (FLIP_A) {
#pragma unroll
      for (int i = 0; i < FM; ++i) a[i] ^= (int)0x80808080u;
    }
    if (SUM_B) {
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumB[j] = __builtin_amdgcn_sdot4(b[j][r], 0x01010101, sumB[j], false);
    }
    if (FLIP_B) {
#pragma unroll
      for (int j = 0; j < FN; ++j) b[j] ^= (int)0x80808080u;
    }
    if (SUM_A) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumA[i] = __builtin_amdgcn_sdot4(a[i][r], 0x01010101, sumA[i], false);
    }
  };

  // block 0 visible to everyone, its first fragments on their way
  if (nkt > 2) publish_barrier<2 * PER_BLOCK>();
  else if (nkt > 1) publish_barrier<PER_BLOCK>();
  else publish_barrier<0>();
#pragma unroll
  for (int f = 0; f < NF; ++f) read_frag(0, 0, f, fa[0], fb[0]);

  // One k block of 64 = two sub-blocks of 32.  The instruction order is pinned
  // (sched_barrier after every slot) so that LDS reads and direct loads sit
  // between MFMAs and their latency hides behind the matrix pipe:
  //   sub-block 0 MFMAs, with the fragment reads of sub-block 1 and, if ISSUE, the
  //                      direct loads of block t+3 (into the stage read in step t-1)
  //   publish barrier    block t+1 becomes visible
  //   sub-block 1 MFMAs, with the fragment reads of block t+1, sub-block 0
  // NEWER: whole blocks that may still be in flight when block t+1 must be
  // complete; -1 marks the last block (nothing to publish).
  constexpr int SLOTS0 = NM > NF + PER_BLOCK ? NM : NF + PER_BLOCK;
  constexpr int SLOTS1 = NM > NF ? NM : NF;
  auto step = [&](int t, auto issue_tag, auto newer_tag) {
    constexpr bool ISSUE = decltype(issue_tag)::value;
    constexpr int NEWER = decltype(newer_tag)::value;
    const int stage = t & (DMA_STAGES - 1);
    const int fill = (t + DMA_STAGES - 1) & (DMA_STAGES - 1);
    const int next = (t + 1) & (DMA_STAGES - 1);
    prepare(fa[0], fb[0]);
#pragma unroll
    for (int s = 0; s < SLOTS0; ++s) {
      if (s < NM)
        acc[s / FN][s % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
            fb[0][s % FN], fa[0][s / FN], acc[s / FN][s % FN], 0, 0, 0);
      if (s < NF) read_frag(stage, 1, s, fa[1], fb[1]);
      else if (ISSUE && s - NF < PER_BLOCK) issue_one(fill, s - NF);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (ISSUE) advance();
    if (NEWER >= 0) publish_barrier<(NEWER > 0 ? NEWER : 0) * PER_BLOCK>();
    prepare(fa[1], fb[1]);
#pragma unroll
    for (int s = 0; s < SLOTS1; ++s) {
      if (s < NM)
        acc[s / FN][s % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
            fb[1][s % FN], fa[1][s / FN], acc[s / FN][s % FN], 0, 0, 0);
      if (NEWER >= 0 && s < NF) read_frag(next, 0, s, fa[0], fb[0]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using std::integral_constant;
  int t = 0;
  for (; t + DMA_STAGES - 1 < nkt; ++t)  // blocks t+1, t+2, t+3 exist; t+2 and t+3 may fly
    step(t, integral_constant<bool, true>{}, integral_constant<int, 2>{});
  // the last (up to) three blocks: nothing left to issue
  if (t + 2 < nkt) { step(t, integral_constant<bool, false>{}, integral_constant<int, 1>{}); ++t; }
  if (t + 1 < nkt) { step(t, integral_constant<bool, false>{}, integral_constant<int, 0>{}); ++t; }
  step(t, integral_constant<bool, false>{}, integral_constant<int, -1>{});

  // ---- write-back: unsigned-operand correction, then C = / += / atomic += ----
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // stages are dead from here on
  // supplied k sums: the lane that would hold the first half of a column's (row's) sum takes
  // the whole of it, its partner 32 lanes on zero
  if (UNS == 3) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int64_t col = n0 + wn * (BN / 2) + j * 32 + (lane & 31);
      sumB[j] = lane < 32 && col < P.n ? P.ksum[col] : 0;
    }
  }
  if (UNS == 4) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int64_t row = m0 + wm * (BM / 2) + i * 32 + (lane & 31);
      sumA[i] = lane < 32 && row < P.m ? P.ksum[row] : 0;
    }
  }
  unsigned_correction<FM, FN>(acc, sumA, sumB, FLIP_A, FLIP_B, lane);
  if (P.slots) {  // only the workgroup that draws the tile's last ticket writes C
    const int64_t tile = ((int64_t)blockIdx.z * P.tiles_m + tm) * P.tiles_n + tn;
    if (!combine_k_ranges<FM, FN>(acc, P.slots + tile * P.splits * (int64_t)(BM * BN), blockIdx.y,
                                  P.splits, P.tickets + tile, wave, lane, tid,
                                  reinterpret_cast<int *>(smem)))
      return;
    __syncthreads();  // the word of LDS the ticket went through is patch memory below
  }
  const int64_t mw = m0 + wm * (BM / 2), nw = n0 + wn * (BN / 2);  // the wave's sub-tile
  if (mw < P.m && nw < P.n) {
    if (P.out_float == 2) {  // int8 output: C is a matrix of bytes
      int8_t *Q = reinterpret_cast<int8_t *>(P.C) + mw * P.ldc + nw;
      if constexpr (FN >= 2) {
        if (m0 + BM <= P.m && n0 + BN <= P.n) {
          store_blocks_q8_via_lds<FM, FN>(acc, Q, P.ldc, lane, smem + wave * STORE_PATCH_BYTES, P.scale);
          return;
        }
      }
      store_blocks_q8<FM, FN>(acc, Q, P.ldc, P.m - mw, P.n - nw, lane, P.scale);
      return;
    }
    int32_t *C = P.C + mw * P.ldc + nw;
    const bool full = m0 + BM <= P.m && n0 + BN <= P.n;
    const Finish fin = {P.scale, P.out_float};
    if (P.atomic)
      add_blocks_atomic<FM, FN>(acc, C, P.ldc, P.m - mw, P.n - nw, lane,
                                reinterpret_cast<int32_t *>(smem + wave * ATOMIC_PATCH_BYTES));
    else if (full)
      store_blocks_via_lds<FM, FN>(acc, C, P.ldc, P.accumulate, lane,
                                   reinterpret_cast<int32_t *>(smem + wave * STORE_PATCH_BYTES), fin);
    else store_blocks<FM, FN, false>(acc, C, P.ldc, P.m - mw, P.n - nw, P.accumulate, lane, fin);
  }
}

template <int BM, int BN>
bool dma_tile_eligible_for(const Problem &p) {
  if (p.k % BK || p.k < BK) return false;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  if (p.conv) {
    const ConvGeom &g = *p.conv;
    if (!a_kc || !b_kc || !p.a_unsigned || g.ci % BK || p.batch != 1) return false;
    const int64_t images = (p.m + (int64_t)g.ho * g.wo - 1) / ((int64_t)g.ho * g.wo);
    if (images * g.hi * g.wi * g.ci >= ((int64_t)1 << 31)) return false;  // 32-bit byte offsets
  }
  const int64_t lda = a_kc ? p.a_sm : p.a_sk;
  const int64_t ldb = b_kc ? p.b_sn : p.b_sk;
  if (lda % 16 || ldb % 16) return false;
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  if (p.batch > 1 && (p.a_sb % 16 || p.b_sb % 16)) return false;  // every problem's operands aligned
  if (!a_kc && p.m % 16) return false;
  if (!b_kc && p.n % 16) return false;
  const int64_t lim = (int64_t)1 << 31;
  if ((a_kc ? BM : BK) * lda + BM >= lim || (b_kc ? BN : BK) * ldb + BN >= lim) return false;
  if (((p.m + BM - 1) / BM) * ((p.n + BN - 1) / BN) > ((int64_t)1 << 30)) return false;
  return true;
}

template <int BM, int BN>
hipError_t launch_dma_tile_for(const Problem &p, int splits, hipStream_t s) {
  DmaTileParams P;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  P.A = static_cast<const uint8_t *>(p.A);
  P.B = static_cast<const uint8_t *>(p.B);
  P.C = p.C;
  P.m = p.m;
  P.n = p.n;
  P.lda = a_kc ? p.a_sm : p.a_sk;
  P.ldb = b_kc ? p.b_sn : p.b_sk;
  P.ldc = p.ldc;
  P.tiles_m = (int)((p.m + BM - 1) / BM);
  P.tiles_n = (int)((p.n + BN - 1) / BN);
  P.nkt = (int)(p.k / BK);
  if (splits < 1) splits = 1;
  if (splits > P.nkt) splits = P.nkt;
  if (splits > 65535) splits = 65535;
  P.kt_per_split = (P.nkt + splits - 1) / splits;
  splits = (P.nkt + P.kt_per_split - 1) / P.kt_per_split;  // no empty ranges
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  const int64_t all_tiles = (int64_t)P.tiles_m * P.tiles_n * (p.batch > 1 ? p.batch : 1);
  P.slots = nullptr;
  P.tickets = nullptr;
  P.splits = splits;
  // A float output cannot add its k ranges into C (float sums must not be combined in
  // arbitrary order): given room for one slot of integer partial sums per k range and tile,
  // the ranges meet there, and the workgroup that comes last converts the complete sum.
  // (An int32 output keeps the atomics: measured on twelve shapes, slots win where C is
  // large, 2048^3 in two ranges 22 against 40 us, but there no split wins at all, 15 us;
  // where splitting pays C is small and the atomics are cheaper, (16, 4096, 4096) in four
  // ranges 8.3 against 9.1 us, (512, 512, 4096) 10.5 against 17 us.)
  if (splits > 1 && p.out_float && p.ws &&
      p.ws_bytes / ((size_t)BM * BN * 4) / (size_t)splits >= (size_t)all_tiles) {
    unsigned *tickets = nullptr;
    if (splitk_tickets(all_tiles, &tickets) == hipSuccess) {
      P.slots = static_cast<int32_t *>(p.ws);
      P.tickets = tickets;
    }
  }
  if (p.out_float && !P.slots) splits = 1;  // float sums must not be combined in arbitrary order
  P.atomic = splits > 1 && !P.slots;
  if (P.atomic && !p.accumulate) {
    hipError_t e = launch_fill_zero(p, s);  // partial sums are added into C: start from zero
    if (e != hipSuccess) return e;
  }
  P.a_sb = p.a_sb;
  P.b_sb = p.b_sb;
  P.c_sb = p.c_sb;
  const int ntiles = P.tiles_m * P.tiles_n;
  if (splits == 1) {  // (a float output that found no room for slots)
    P.kt_per_split = P.nkt;
    P.splits = 1;
  }
  // a workgroup with fewer k blocks than stages never touches the later stages: leave them
  // out, so that more workgroups of a short-k problem fit a compute unit (the write-back
  // patches, one per wave, must still fit)
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8), (unsigned)splits, (unsigned)p.batch);
  const int stages = P.kt_per_split < DMA_STAGES ? P.kt_per_split : DMA_STAGES;
  size_t lds = (size_t)stages * (BM + BN) * BK;
  if (lds < 4 * (size_t)STORE_PATCH_BYTES) lds = 4 * (size_t)STORE_PATCH_BYTES;
  const int uns = p.a_unsigned ? 1 : (p.b_unsigned ? 2 : 0);
  // supplied k sums (pre-packed weights): for an unsplit k and a k-contiguous signed operand,
  // which packed weights always are; otherwise the sums are accumulated in the loop as usual
  const bool supplied = p.ksum != nullptr && splits == 1 && p.batch <= 1 && !p.conv &&
                        ((uns == 1 && b_kc) || (uns == 2 && a_kc));
  P.ksum = supplied ? p.ksum : nullptr;
  void (*kern)(DmaTileParams) = nullptr;
#define MIP_PICK(AK, BKC)                                                          \
  kern = uns == 0 ? dma_tile_kernel<BM, BN, AK, BKC, 0>                            \
                  : (uns == 1 ? dma_tile_kernel<BM, BN, AK, BKC, 1>                \
                              : dma_tile_kernel<BM, BN, AK, BKC, 2>)
  if (supplied && uns == 1)
    kern = a_kc ? dma_tile_kernel<BM, BN, true, true, 3> : dma_tile_kernel<BM, BN, false, true, 3>;
  else if (supplied)
    kern = b_kc ? dma_tile_kernel<BM, BN, true, true, 4> : dma_tile_kernel<BM, BN, true, false, 4>;
  else if (a_kc && b_kc) MIP_PICK(true, true);
  else if (a_kc) MIP_PICK(true, false);
  else if (b_kc) MIP_PICK(false, true);
  else MIP_PICK(false, false);
#undef MIP_PICK
  if (p.conv) {
    P.conv = *p.conv;
    // (the gathered matrix is the unsigned A, the filters the signed, k-contiguous B)
    const bool filter_sums = p.ksum != nullptr && splits == 1;
    P.ksum = filter_sums ? p.ksum : nullptr;
    kern = filter_sums ? dma_tile_kernel<BM, BN, true, true, 3, true> : dma_tile_kernel<BM, BN, true, true, 1, true>;
  } else {
    P.conv = ConvGeom{};
  }
  {
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds, s, P);
  return hipGetLastError();
}

}  // namespace mip
