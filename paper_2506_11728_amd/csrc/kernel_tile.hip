// MFMA tile kernels for the MIP GEMM on gfx950.
//
// Roles taken from the paper's algorithm (Section 3, figure "Reference GEMM
// algorithm", and Section 4.1), re-cast for a GPU:
//   loops L1/L3 (jc, ic over n, m)  ->  the grid: one workgroup per BM x BN tile of C
//   loop  L2    (pc over k)         ->  the K loop of a workgroup, BK = 64 per step
//   Pack A / Pack B                 ->  staging of a BM x BK block of A and a BK x BN block
//                                       of B into LDS, in an order from which every lane
//                                       fetches 16 consecutive k per operand register;
//                                       storage order, leading dimension and the
//                                       unsigned-operand bias are absorbed here
//   loops L4/L5 (jr, ir)            ->  the 2 x 2 waves of a workgroup and the 32 x 32 blocks
//                                       of each wave's sub-tile
//   micro-kernel, loop L6           ->  v_mfma_i32_32x32x32_i8 on register-resident int32
//                                       accumulators (C_r), written back once after the K loop
//
// v_mfma_i32_32x32x32_i8 lane layout (measured on the device):
//   operand a: lane l holds row (l % 32), 16 consecutive k starting at 16 * (l / 32)
//   operand b: lane l holds column (l % 32), same 16 k
//   result   : lane l holds column (l % 32); register v holds row 8*(v/4) + 4*(l/32) + v%4
// The kernels pass the B fragment as operand a and the A fragment as operand b, so the
// block comes out transposed: lane = row of C, four consecutive registers = four
// consecutive columns, which makes the write-back one 16-byte store per lane.
//
// Unsigned operands: the matrix instruction multiplies signed bytes only.  An
// unsigned x is staged as the signed byte x - 128 (x ^ 0x80), and the epilogue
// adds 128 * sum_p y(p) of the other (signed) operand, which the waves
// accumulate from the fragments they already hold.  Exact modulo 2^32.
#include "epilogue.h"
#include "lds_layout.h"
#include "mip_internal.h"

namespace mip {

struct TileParams {
  Problem p;
  int tiles_m, tiles_n;
  int kt_per_split;  // k blocks of 64 handled by one workgroup (blockIdx.y picks the range)
  int atomic;        // several workgroups add into the same tile of C (split k)
};

template <int BM, int BN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHREADS) void tile_kernel(TileParams tp) {
  constexpr int FM = BM / 64, FN = BN / 64;  // 32 x 32 blocks per wave, down and across
  using SA = Stage<BM, A_KC>;
  using SB = Stage<BN, B_KC>;
  constexpr int STAGE_BYTES = (BM + BN) * BK;
  // two operand stages; the split-k write-back reuses the space as four transpose patches
  constexpr int SMEM_BYTES =
      2 * STAGE_BYTES > 4 * STORE_PATCH_BYTES ? 2 * STAGE_BYTES : 4 * STORE_PATCH_BYTES;
  __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM_BYTES];

  Problem p = tp.p;
  {  // problem of the batch
    const int64_t z = blockIdx.z;
    p.A = static_cast<const uint8_t *>(p.A) + z * p.a_sb;
    p.B = static_cast<const uint8_t *>(p.B) + z * p.b_sb;
    p.C += z * p.c_sb;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of
  // them, each with its own L2), so give every XCD a contiguous run of tiles,
  // and walk the tiles in groups of 8 tile-rows so that the workgroups resident
  // on one XCD share A row-panels and B column-panels.
  const int ntiles = tp.tiles_m * tp.tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  int lid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (lid >= ntiles) return;
  constexpr int GROUP = 8;
  const int per_group = GROUP * tp.tiles_n;
  const int first_m = (lid / per_group) * GROUP;
  const int gsz = tp.tiles_m - first_m < GROUP ? tp.tiles_m - first_m : GROUP;
  const int tm = first_m + (lid % per_group) % gsz;
  const int tn = (lid % per_group) / gsz;

  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const uint8_t *A = static_cast<const uint8_t *>(p.A);
  const uint8_t *B = static_cast<const uint8_t *>(p.B);
  const int flipA = p.a_unsigned ? (int)0x80808080u : 0;
  const int flipB = p.b_unsigned ? (int)0x80808080u : 0;

  // Split k: integer addition is associative, so partial sums added into C in
  // any order give the same bits as one pass.
  const int64_t nkt = (p.k + BK - 1) / BK;  // k blocks in the whole problem
  const int64_t kt_begin = (int64_t)blockIdx.y * tp.kt_per_split;
  const int64_t kt_end = kt_begin + tp.kt_per_split < nkt ? kt_begin + tp.kt_per_split : nkt;
  if (kt_begin >= kt_end) return;
  const bool edge_tile = m0 + BM > p.m || n0 + BN > p.n;
  const bool k_tail = (p.k % BK) != 0;

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

  v4i ra[SA::PER_THREAD], rb[SB::PER_THREAD];

  auto load_block = [&](int64_t kt) {
    const bool checked = edge_tile || (k_tail && kt == nkt - 1);
    if (!checked) {
      SA::template load<false>(ra, A, p.a_sm, p.a_sk, m0, kt * BK, p.m, p.k, tid, flipA);
      SB::template load<false>(rb, B, p.b_sn, p.b_sk, n0, kt * BK, p.n, p.k, tid, flipB);
    } else {
      SA::template load<true>(ra, A, p.a_sm, p.a_sk, m0, kt * BK, p.m, p.k, tid, flipA);
      SB::template load<true>(rb, B, p.b_sn, p.b_sk, n0, kt * BK, p.n, p.k, tid, flipB);
    }
  };
  auto store_block = [&](int stage) {
    uint8_t *sa = smem + stage * STAGE_BYTES;
    SA::store(ra, sa, tid);
    SB::store(rb, sa + BM * BK, tid);
  };

  load_block(kt_begin);
  store_block(0);
  __syncthreads();

  for (int64_t kt = kt_begin; kt < kt_end; ++kt) {
    const int stage = (int)((kt - kt_begin) & 1);
    if (kt + 1 < kt_end) load_block(kt + 1);

    const uint8_t *sa = smem + stage * STAGE_BYTES;
    const uint8_t *sb = sa + BM * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      v4i fa[FM], fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[i] = SA::fragment(sa, wm * (BM / 2) + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[j] = SB::fragment(sb, wn * (BN / 2) + j * 32, ks, lane);
      if (flipA) {  // A unsigned: need sum over k of B's columns
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            sumB[j] = __builtin_amdgcn_sdot4(fb[j][r], 0x01010101, sumB[j], false);
      }
      if (flipB) {  // B unsigned: need sum over k of A's rows
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            sumA[i] = __builtin_amdgcn_sdot4(fa[i][r], 0x01010101, sumA[i], false);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }

    if (kt + 1 < kt_end) store_block(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: unsigned-operand correction, then C = acc or C += acc ----
  unsigned_correction<FM, FN>(acc, sumA, sumB, flipA != 0, flipB != 0, lane);
  const int64_t mw = m0 + wm * (BM / 2), nw = n0 + wn * (BN / 2);  // the wave's sub-tile
  if (mw < p.m && nw < p.n) {
    if (p.out_float == 2) {  // int8 output: C is a matrix of bytes
      int8_t *Q = reinterpret_cast<int8_t *>(p.C) + mw * p.ldc + nw;
      if constexpr (FN >= 2) {
        if (!edge_tile) {
          // the k loop ended on a workgroup barrier: no wave still reads the stages
          store_blocks_q8_via_lds<FM, FN>(acc, Q, p.ldc, lane, smem + wave * STORE_PATCH_BYTES, p.scale);
          return;
        }
      }
      store_blocks_q8<FM, FN>(acc, Q, p.ldc, p.m - mw, p.n - nw, lane, p.scale);
      return;
    }
    int32_t *C = p.C + mw * p.ldc + nw;
    const Finish fin = {p.scale, p.out_float};
    if (tp.atomic) {
      // the k loop ended on a workgroup barrier: no wave still reads the stages
      add_blocks_atomic<FM, FN>(acc, C, p.ldc, p.m - mw, p.n - nw, lane,
                                reinterpret_cast<int32_t *>(smem + wave * ATOMIC_PATCH_BYTES));
    }
    else if (!edge_tile)
      store_blocks_via_lds<FM, FN>(acc, C, p.ldc, p.accumulate, lane,
                                   reinterpret_cast<int32_t *>(smem + wave * STORE_PATCH_BYTES), fin);
    else store_blocks<FM, FN, false>(acc, C, p.ldc, p.m - mw, p.n - nw, p.accumulate, lane, fin);
  }
}

template <int BM, int BN>
static hipError_t launch_cfg(const Problem &p, int splits, hipStream_t s) {
  TileParams tp;
  tp.p = p;
  int64_t tiles_m = (p.m + BM - 1) / BM, tiles_n = (p.n + BN - 1) / BN;
  if (tiles_m * tiles_n > (int64_t)1 << 30) return hipErrorInvalidValue;
  tp.tiles_m = (int)tiles_m;
  tp.tiles_n = (int)tiles_n;
  const int64_t nkt = (p.k + BK - 1) / BK;
  if (splits < 1 || p.out_float) splits = 1;  // float sums must not be combined in arbitrary order
  if (splits > nkt) splits = (int)nkt;
  if (splits > 65535) splits = 65535;
  tp.kt_per_split = (int)((nkt + splits - 1) / splits);
  splits = (int)((nkt + tp.kt_per_split - 1) / tp.kt_per_split);  // no empty ranges
  tp.atomic = splits > 1;
  if (tp.atomic && !p.accumulate) {
    // partial sums are added into C: start it from zero
    hipError_t e = launch_fill_zero(p, s);
    if (e != hipSuccess) return e;
  }
  int ntiles = tp.tiles_m * tp.tiles_n;
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8), (unsigned)splits, (unsigned)p.batch);
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  if (a_kc && b_kc) hipLaunchKernelGGL((tile_kernel<BM, BN, true, true>), grid, dim3(NTHREADS), 0, s, tp);
  else if (a_kc) hipLaunchKernelGGL((tile_kernel<BM, BN, true, false>), grid, dim3(NTHREADS), 0, s, tp);
  else if (b_kc) hipLaunchKernelGGL((tile_kernel<BM, BN, false, true>), grid, dim3(NTHREADS), 0, s, tp);
  else hipLaunchKernelGGL((tile_kernel<BM, BN, false, false>), grid, dim3(NTHREADS), 0, s, tp);
  return hipGetLastError();
}

hipError_t launch_staged(const Problem &p, Shape shape, int splits, hipStream_t s) {
  switch (shape) {
    case SHAPE_256: return launch_cfg<256, 256>(p, splits, s);
    case SHAPE_128: return launch_cfg<128, 128>(p, splits, s);
    case SHAPE_64: return launch_cfg<64, 64>(p, splits, s);
    case SHAPE_64X256: return launch_cfg<64, 256>(p, splits, s);
    case SHAPE_256X64: return launch_cfg<256, 64>(p, splits, s);
    case SHAPE_64X128: return launch_cfg<64, 128>(p, splits, s);
    case SHAPE_128X64: return launch_cfg<128, 64>(p, splits, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mip
