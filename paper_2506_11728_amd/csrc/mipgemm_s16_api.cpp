// C-ABI entry point of the product with 16-bit operands: the operands are split into byte
// planes, three 8-bit GEMMs of this library run on them, and one kernel puts the pieces
// together (kernel_s16.hip).  Host only.
#include "api_internal.h"

using mip::order_ok;

namespace {

int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

// The workspace of a call, every part a multiple of 256 bytes: the planes of A (m rows of
// 2 kp bytes) and of B (n rows), four vectors of plane sums, three dense m x n int32 products.
struct S16Layout {
  int64_t kp;
  size_t planes_a, planes_b, sums, product, total;
};
bool s16_layout(int64_t m, int64_t n, int64_t k, S16Layout *L) {
  if (m < 0 || n < 0 || k < 0 || m > MIPGEMM_MAX_DIM || n > MIPGEMM_MAX_DIM || k > MIPGEMM_MAX_DIM)
    return false;
  L->kp = k >= 1024 ? round_up(k, 128) : round_up(k > 0 ? k : 1, 64);
  if (2 * L->kp > MIPGEMM_MAX_DIM) return false;
  const double bytes = 2.0 * (double)L->kp * ((double)m + (double)n) + 12.0 * (double)m * (double)n;
  if (bytes > 4.0e18) return false;
  L->planes_a = (size_t)round_up(m * 2 * L->kp, 256);
  L->planes_b = (size_t)round_up(n * 2 * L->kp, 256);
  L->sums = (size_t)round_up((2 * m + 2 * n + 4) * 4, 256);
  L->product = (size_t)round_up(m * n * 4, 256);
  L->total = L->planes_a + L->planes_b + L->sums + 3 * L->product;
  return true;
}

}  // namespace

extern "C" {

size_t mipgemm_workspace_size_s16(int64_t m, int64_t n, int64_t k) {
  S16Layout L;
  if (!s16_layout(m, n, k, &L) || m == 0 || n == 0 || k == 0) return 0;
  return L.total + 256;  // room to align the start
}

int mipgemm_s16s16s32(int64_t m, int64_t n, int64_t k, const int16_t *A, int64_t lda, int orderA,
                      const int16_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                      int mode, void *workspace, size_t workspace_bytes, void *stream) {
  if (m < 0 || m > MIPGEMM_MAX_DIM) return -1;
  if (n < 0 || n > MIPGEMM_MAX_DIM) return -2;
  if (k < 0 || k > MIPGEMM_MAX_DIM) return -3;
  if (!A && m > 0 && k > 0) return -4;
  if (!order_ok(orderA)) return -6;
  {
    const int64_t need = orderA == MIPGEMM_ROW_MAJOR ? k : m;
    if (lda < (need > 1 ? need : 1) || lda > MIPGEMM_MAX_DIM) return -5;
  }
  if (!B && k > 0 && n > 0) return -7;
  if (!order_ok(orderB)) return -9;
  {
    const int64_t need = orderB == MIPGEMM_ROW_MAJOR ? n : k;
    if (ldb < (need > 1 ? need : 1) || ldb > MIPGEMM_MAX_DIM) return -8;
  }
  if (!C && m > 0 && n > 0) return -10;
  if (!order_ok(orderC)) return -12;
  {
    const int64_t need = orderC == MIPGEMM_ROW_MAJOR ? n : m;
    if (ldc < (need > 1 ? need : 1) || ldc > MIPGEMM_MAX_DIM) return -11;
  }
  if (mode != MIPGEMM_OVERWRITE && mode != MIPGEMM_ACCUMULATE) return -13;
  if (workspace_bytes > 0 && !workspace) return -14;
  if (m == 0 || n == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool accumulate = mode == MIPGEMM_ACCUMULATE;

  // a column-major C (m x n) is the row-major C^T (n x m) = B^T A^T on the same memory
  int64_t rm = m, rn = n;
  const int16_t *X = A, *Y = B;  // X: the operand whose rows are the rows of the row-major C
  int64_t x_sr = orderA == MIPGEMM_ROW_MAJOR ? lda : 1, x_sk = orderA == MIPGEMM_ROW_MAJOR ? 1 : lda;
  int64_t y_sr = orderB == MIPGEMM_ROW_MAJOR ? 1 : ldb, y_sk = orderB == MIPGEMM_ROW_MAJOR ? ldb : 1;
  if (orderC != MIPGEMM_ROW_MAJOR) {
    rm = n; rn = m;
    X = B; Y = A;
    const int64_t sr = x_sr, sk = x_sk;
    x_sr = y_sr; x_sk = y_sk;
    y_sr = sr; y_sk = sk;
  }
  if (k == 0) {  // an empty sum: overwrite stores zeros, accumulate leaves C alone
    if (accumulate) return 0;
    mip::Problem z;
    z.m = rm; z.n = rn; z.k = 0; z.C = C; z.ldc = ldc;
    return static_cast<int>(mip::launch_fill_zero(z, s));
  }
  S16Layout L;
  if (!s16_layout(rm, rn, k, &L)) return -3;
  if (!workspace) return -14;
  uint8_t *ws = static_cast<uint8_t *>(workspace);
  const size_t skip = (256 - reinterpret_cast<uintptr_t>(ws) % 256) % 256;
  if (workspace_bytes < skip + L.total) return -15;
  ws += skip;
  uint8_t *PA = ws, *PB = PA + L.planes_a;
  int32_t *sums = reinterpret_cast<int32_t *>(PB + L.planes_b);
  int32_t *sA = sums, *sB = sums + 2 * rm + (2 * rm % 4 ? 4 - 2 * rm % 4 : 0);  // (16-byte aligned)
  int32_t *T1 = reinterpret_cast<int32_t *>(reinterpret_cast<uint8_t *>(sums) + L.sums);
  int32_t *T2 = reinterpret_cast<int32_t *>(reinterpret_cast<uint8_t *>(T1) + L.product);
  int32_t *T3 = reinterpret_cast<int32_t *>(reinterpret_cast<uint8_t *>(T2) + L.product);
  const int64_t kp = L.kp;

  hipError_t e = mip::launch_split_planes(X, x_sr, x_sk, rm, k, kp, PA, true, s);   // [ah | al]
  if (e != hipSuccess) return static_cast<int>(e);
  e = mip::launch_split_planes(Y, y_sr, y_sk, rn, k, kp, PB, false, s);              // [bl | bh]
  if (e != hipSuccess) return static_cast<int>(e);
  // a row of 2 kp bytes is two columns of kp: one launch per operand sums both planes of every row
  e = mip::launch_column_sums(kp, 2 * rm, PA, kp, sA, s);
  if (e == hipSuccess) e = mip::launch_column_sums(kp, 2 * rn, PB, kp, sB, s);
  if (e != hipSuccess) return static_cast<int>(e);
  // the three byte products, each an s8 x s8 GEMM of this library on the planes
  const int R = MIPGEMM_ROW_MAJOR, Cm = MIPGEMM_COL_MAJOR, OVW = MIPGEMM_OVERWRITE;
  int rc = mip::run_gemm(0, 0, 0, 1.0f, rm, rn, kp, PA, 2 * kp, R, PB + kp, 2 * kp, Cm, T1, rn, R, OVW,
                         nullptr, 0, stream);                                   // ah bh
  if (rc == 0)
    rc = mip::run_gemm(0, 0, 0, 1.0f, rm, rn, 2 * kp, PA, 2 * kp, R, PB, 2 * kp, Cm, T2, rn, R, OVW,
                       nullptr, 0, stream);                                     // ah bl + al bh
  if (rc == 0)
    rc = mip::run_gemm(0, 0, 0, 1.0f, rm, rn, kp, PA + kp, 2 * kp, R, PB, 2 * kp, Cm, T3, rn, R, OVW,
                       nullptr, 0, stream);                                     // al bl
  if (rc != 0) return rc > 0 ? rc : static_cast<int>(hipErrorInvalidValue);  // (sizes were checked above)
  return static_cast<int>(mip::launch_combine_planes(T1, T2, T3, sA, sB, rm, rn, k, C, ldc,
                                                     accumulate, s));
}

}  // extern "C"
