// Launchers of the kernel with 128-deep k blocks (dma_k128.h): the 256 x 256 form for large,
// aligned problems and the 128 x 128 form on whole tiles.
#include "dma_k128.h"

namespace mip {

// small: the 128 x 128 form (whole tiles only)
bool dma_k128_eligible(const Problem &p, bool small) {
  if (p.conv || p.batch != 1 || p.k % KD2 || p.k < KD2) return false;
  if (small) {
    if (p.m % 128 || p.n % 128) return false;
  } else if ((p.m % DM || p.n % DN) && !(p.rows_padded_to_256 && p.a_sk == 1 && p.b_sk == 1)) {
    return false;  // ragged m or n: only on k-contiguous operands padded to whole tiles of rows
  }
  const int64_t lda = p.a_sk == 1 ? p.a_sm : p.a_sk;
  const int64_t ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  if (lda % 16 || ldb % 16) return false;
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  if (256 * lda >= ((int64_t)1 << 31) || 256 * ldb >= ((int64_t)1 << 31)) return false;
  const int64_t bm = small ? 128 : DM, bn = small ? 128 : DN;
  if (((p.m + bm - 1) / bm) * ((p.n + bn - 1) / bn) > ((int64_t)1 << 30)) return false;
  return true;
}

namespace {

template <int BM, int BN>
hipError_t launch_for(const Problem &p, hipStream_t s, unsigned long long *clocks) {
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
  P.tiles_m = (int)((p.m + BM - 1) / BM);
  P.tiles_n = (int)((p.n + BN - 1) / BN);
  P.nkt = (int)(p.k / KD2);
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  P.splits = 1;
  P.atomic = 0;
  const int ntiles = P.tiles_m * P.tiles_n;
  dim3 grid((unsigned)(((ntiles + 7) / 8) * 8));
  // (measured at 8192^3, four rounds: 326 -> 310 us on constant operands, 452 -> 444 us on
  // random ones; the 7 us of late start are not earned back by a single round; the 128 x 128
  // form, two workgroups to a compute unit and a short write-back, starts all at once)
  P.first_round = (int)compute_units();
  P.stagger_ticks = BM == DM && ntiles >= 2 * P.first_round ? STAGGER_TICKS : 0;
  if (tuning().stagger >= 0 && BM == DM) P.stagger_ticks = tuning().stagger;  // tuning runs
  const size_t lds = (size_t)Tile16<BM, BN>::LDS_BYTES;
  const bool a_kc = p.a_sk == 1, b_kc = p.b_sk == 1;
  const int uns = p.a_unsigned ? 1 : (p.b_unsigned ? 2 : 0);
  // supplied k sums (pre-packed weights): instantiated for a k-contiguous signed operand,
  // which packed weights always are; otherwise the sums are accumulated in the loop as usual
  const bool supplied = p.ksum != nullptr && ((uns == 1 && b_kc) || (uns == 2 && a_kc));
  P.ksum = supplied ? p.ksum : nullptr;
  void (*kern)(DmaParams) = nullptr;
#define MIP_PICK(AK, BKC)                                                                    \
  kern = uns == 0 ? dma128_kernel<BM, BN, AK, BKC, 0>                                        \
                  : (uns == 1 ? dma128_kernel<BM, BN, AK, BKC, 1> : dma128_kernel<BM, BN, AK, BKC, 2>)
  if (BM == DM && (p.m % DM || p.n % DN))
    kern = uns == 0 ? dma128_kernel<DM, DN, true, true, 0, true>
           : supplied ? (uns == 1 ? dma128_kernel<DM, DN, true, true, 3, true>
                                  : dma128_kernel<DM, DN, true, true, 4, true>)
                      : (uns == 1 ? dma128_kernel<DM, DN, true, true, 1, true>
                                  : dma128_kernel<DM, DN, true, true, 2, true>);
  else if (supplied && uns == 1)
    kern = a_kc ? dma128_kernel<BM, BN, true, true, 3> : dma128_kernel<BM, BN, false, true, 3>;
  else if (supplied)
    kern = b_kc ? dma128_kernel<BM, BN, true, true, 4> : dma128_kernel<BM, BN, true, false, 4>;
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

}  // namespace

hipError_t launch_dma_k128(const Problem &p, hipStream_t s, unsigned long long *clocks, bool small) {
  return small ? launch_for<128, 128>(p, s, clocks) : launch_for<DM, DN>(p, s, clocks);
}

}  // namespace mip
