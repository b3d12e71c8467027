// The kernel with 128-deep k blocks (dma_k128.h) in its general form: ragged m and n on
// unpadded operands, on 256 x 256 or 128 x 128 tiles; on the latter k may be cut into ranges,
// for problems whose tiles are too few to occupy the device while k is long: every range of a
// tile is a workgroup of its own, and the ranges add their partial sums into C with integer
// atomics.
#include "dma_k128.h"

namespace mip {

bool dma_k128_split_eligible(const Problem &p, bool large) {
  if (p.conv || p.batch != 1 || p.k % KD2 || p.k < KD2) return false;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  if (!a_kc && (p.a_sm != 1 || p.m % 16)) return false;  // a strided operand comes in 16-byte chunks
  if (!b_kc && (p.b_sn != 1 || p.n % 16)) return false;
  const int64_t lda = a_kc ? p.a_sm : p.a_sk;
  const int64_t ldb = b_kc ? p.b_sn : p.b_sk;
  if (lda % 16 || ldb % 16) return false;
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  const int64_t side = large ? 256 : 128;
  if (side * lda >= ((int64_t)1 << 31) || side * ldb >= ((int64_t)1 << 31)) return false;
  if (((p.m + side - 1) / side) * ((p.n + side - 1) / side) > ((int64_t)1 << 30)) return false;
  return true;
}

namespace {

template <int BM, int BN>
hipError_t launch_general(const Problem &p, int splits, hipStream_t s) {
  DmaParams P;
  P.clocks = nullptr;
  P.A = static_cast<const uint8_t *>(p.A);
  P.B = static_cast<const uint8_t *>(p.B);
  P.C = p.C;
  P.lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  P.ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  P.ldc = p.ldc;
  P.m = p.m;
  P.n = p.n;
  P.tiles_m = (int)((p.m + BM - 1) / BM);
  P.tiles_n = (int)((p.n + BN - 1) / BN);
  P.nkt = (int)(p.k / KD2);
  // k ranges on the small tile only, and only into an int32 C (float sums must not be combined
  // in arbitrary order, and an int8 C holds no partial sums)
  if (splits < 1 || BM != 128 || p.out_float) splits = 1;
  if (splits > P.nkt) splits = P.nkt;       // every range holds at least one block
  if (splits > 65535) splits = 65535;
  P.splits = splits;
  P.atomic = splits > 1;
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  P.ksum = nullptr;
  const int ntiles = P.tiles_m * P.tiles_n;
  P.first_round = (int)compute_units();
  // (the large tile's rows of an XCD's patch start apart, as in the form for whole tiles)
  P.stagger_ticks = BM == 256 && ntiles >= 2 * P.first_round ? STAGGER_TICKS : 0;
  if (P.atomic && !p.accumulate) {
    hipError_t e = launch_fill_zero(p, s);  // partial sums are added into C: start from zero
    if (e != hipSuccess) return e;
  }
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8), (unsigned)splits);
  const size_t lds = (size_t)Tile16<BM, BN>::LDS_BYTES;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  const int uns = p.a_unsigned ? 1 : (p.b_unsigned ? 2 : 0);
  void (*kern)(DmaParams) = nullptr;
#define MIP_PICK(AK, BKC)                                                                     \
  kern = uns == 0 ? dma128_kernel<BM, BN, AK, BKC, 0, true, true>                             \
                  : (uns == 1 ? dma128_kernel<BM, BN, AK, BKC, 1, true, true>                 \
                              : dma128_kernel<BM, BN, AK, BKC, 2, true, true>)
  if (a_kc && b_kc) MIP_PICK(true, true);
  else if (a_kc) MIP_PICK(true, false);
  else if (b_kc) MIP_PICK(false, true);
  else MIP_PICK(false, false);
#undef MIP_PICK
  hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds, s, P);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_dma_k128_split(const Problem &p, int splits, hipStream_t s, bool large) {
  return large ? launch_general<256, 256>(p, 1, s) : launch_general<128, 128>(p, splits, s);
}

}  // namespace mip
