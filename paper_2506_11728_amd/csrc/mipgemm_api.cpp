// C-ABI layer of mipgemm: argument validation, normalisation of the storage
// orders and dispatch to the HIP kernels.  Everything here runs on the host.
#include "../../include/mipgemm.h"

#include <cstdlib>
#include <cstring>

#include "mip_internal.h"

namespace mip {

const char *variant_name(Variant v) {
  switch (v) {
    case VARIANT_NONE: return "none";
    case VARIANT_FILL: return "fill_zero";
    case VARIANT_SIMPLE: return "simple";
    case VARIANT_DMA256: return "mfma_dma256";
    case VARIANT_DMA256K128: return "mfma_dma256_k128";
    case VARIANT_TILE256: return "mfma_tile256";
    case VARIANT_TILE128: return "mfma_tile128";
    case VARIANT_TILE64: return "mfma_tile64";
    default: return "?";
  }
}

// MIPGEMM_VARIANT=simple|dma256|tile256|tile128|tile64 pins the kernel (tuning and tests).
// dma256 only applies to problems it is eligible for; others keep the automatic choice.
static Variant forced_variant() {
  const char *e = std::getenv("MIPGEMM_VARIANT");
  if (!e || !*e) return VARIANT_NONE;
  if (!std::strcmp(e, "simple")) return VARIANT_SIMPLE;
  if (!std::strcmp(e, "dma256")) return VARIANT_DMA256;
  if (!std::strcmp(e, "dma256k128")) return VARIANT_DMA256K128;
  if (!std::strcmp(e, "tile256")) return VARIANT_TILE256;
  if (!std::strcmp(e, "tile128")) return VARIANT_TILE128;
  if (!std::strcmp(e, "tile64")) return VARIANT_TILE64;
  return VARIANT_NONE;
}

Variant choose_variant(const Problem &p) {
  if (p.m == 0 || p.n == 0) return VARIANT_NONE;
  if (p.k == 0) return p.accumulate ? VARIANT_NONE : VARIANT_FILL;
  Variant f = forced_variant();
  if (f == VARIANT_DMA256 && !dma_eligible(p, false)) f = VARIANT_NONE;
  if (f == VARIANT_DMA256K128 && !dma_eligible(p, true)) f = VARIANT_NONE;
  if (f != VARIANT_NONE) return f;
  // Tile choice: the largest tile that still yields about one workgroup per
  // compute unit (256 of them); small problems take small tiles.
  auto tiles = [&](int64_t t) { return ((p.m + t - 1) / t) * ((p.n + t - 1) / t); };
  if (tiles(256) >= 192) return dma_eligible(p, false) ? VARIANT_DMA256 : VARIANT_TILE256;
  if (tiles(128) >= 192) return VARIANT_TILE128;
  return VARIANT_TILE64;
}

}  // namespace mip

namespace {

using mip::Problem;

bool order_ok(int o) { return o == MIPGEMM_ROW_MAJOR || o == MIPGEMM_COL_MAJOR; }

// Fills `out` and returns 0, or returns the negative argument number.
int validate_and_normalise(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k,
                           const void *A, int64_t lda, int orderA, const void *B, int64_t ldb,
                           int orderB, int32_t *C, int64_t ldc, int orderC, int mode,
                           void *workspace, size_t workspace_bytes, Problem *out) {
  if (m < 0 || m > MIPGEMM_MAX_DIM) return -1;
  if (n < 0 || n > MIPGEMM_MAX_DIM) return -2;
  if (k < 0 || k > MIPGEMM_MAX_DIM) return -3;
  if (!A && m > 0 && k > 0) return -4;
  if (!order_ok(orderA)) return -6;
  {
    int64_t need = orderA == MIPGEMM_ROW_MAJOR ? k : m;
    if (lda < (need > 1 ? need : 1) || lda > MIPGEMM_MAX_DIM) return -5;
  }
  if (!B && k > 0 && n > 0) return -7;
  if (!order_ok(orderB)) return -9;
  {
    int64_t need = orderB == MIPGEMM_ROW_MAJOR ? n : k;
    if (ldb < (need > 1 ? need : 1) || ldb > MIPGEMM_MAX_DIM) return -8;
  }
  if (!C && m > 0 && n > 0) return -10;
  if (!order_ok(orderC)) return -12;
  {
    int64_t need = orderC == MIPGEMM_ROW_MAJOR ? n : m;
    if (ldc < (need > 1 ? need : 1) || ldc > MIPGEMM_MAX_DIM) return -11;
  }
  if (mode != MIPGEMM_OVERWRITE && mode != MIPGEMM_ACCUMULATE) return -13;
  size_t need_ws = mipgemm_workspace_size(m, n, k, orderA, orderB, orderC);
  if (need_ws > 0 && !workspace) return -14;
  if (workspace_bytes < need_ws) return -15;

  const int64_t a_sm = orderA == MIPGEMM_ROW_MAJOR ? lda : 1;
  const int64_t a_sk = orderA == MIPGEMM_ROW_MAJOR ? 1 : lda;
  const int64_t b_sk = orderB == MIPGEMM_ROW_MAJOR ? ldb : 1;
  const int64_t b_sn = orderB == MIPGEMM_ROW_MAJOR ? 1 : ldb;
  Problem p;
  if (orderC == MIPGEMM_ROW_MAJOR) {
    p.m = m; p.n = n;
    p.A = A; p.a_sm = a_sm; p.a_sk = a_sk; p.a_unsigned = a_unsigned;
    p.B = B; p.b_sk = b_sk; p.b_sn = b_sn; p.b_unsigned = b_unsigned;
  } else {
    // column-major C (m x n) is the row-major C^T (n x m) = B^T A^T on the same memory
    p.m = n; p.n = m;
    p.A = B; p.a_sm = b_sn; p.a_sk = b_sk; p.a_unsigned = b_unsigned;
    p.B = A; p.b_sk = a_sk; p.b_sn = a_sm; p.b_unsigned = a_unsigned;
  }
  p.k = k;
  p.C = C;
  p.ldc = ldc;
  p.accumulate = mode == MIPGEMM_ACCUMULATE;
  *out = p;
  return 0;
}

int run(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k, const void *A,
        int64_t lda, int orderA, const void *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc,
        int orderC, int mode, void *workspace, size_t workspace_bytes, void *stream) {
  Problem p;
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB,
                                  C, ldc, orderC, mode, workspace, workspace_bytes, &p);
  if (rc != 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  mip::Variant v = mip::choose_variant(p);
  switch (v) {
    case mip::VARIANT_NONE: break;
    case mip::VARIANT_FILL: e = mip::launch_fill_zero(p, s); break;
    case mip::VARIANT_SIMPLE: e = mip::launch_simple(p, s); break;
    case mip::VARIANT_DMA256: e = mip::launch_dma(p, false, s); break;
    case mip::VARIANT_DMA256K128: e = mip::launch_dma(p, true, s); break;
    default: e = mip::launch_tile(p, v, s); break;
  }
  return static_cast<int>(e);
}

}  // namespace

extern "C" {

int mipgemm_s8s8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_u8s8s32(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(1, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_s8u8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(0, 1, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

size_t mipgemm_workspace_size(int64_t, int64_t, int64_t, int, int, int) {
  // No kernel stages anything outside A, B and C: operands go straight from
  // their own storage through LDS into the matrix cores.
  return 0;
}

const char *mipgemm_strerror(int code) {
  static const char *const args[] = {
      "success",
      "invalid argument 1 (m)", "invalid argument 2 (n)", "invalid argument 3 (k)",
      "invalid argument 4 (A is null)", "invalid argument 5 (lda too small)",
      "invalid argument 6 (orderA)", "invalid argument 7 (B is null)",
      "invalid argument 8 (ldb too small)", "invalid argument 9 (orderB)",
      "invalid argument 10 (C is null)", "invalid argument 11 (ldc too small)",
      "invalid argument 12 (orderC)", "invalid argument 13 (mode)",
      "invalid argument 14 (workspace is null)",
      "invalid argument 15 (workspace_bytes too small)", "invalid argument 16 (stream)"};
  if (code <= 0 && code >= -16) return args[-code];
  if (code > 0) return hipGetErrorString(static_cast<hipError_t>(code));
  return "unknown mipgemm error code";
}

const char *mipgemm_variant_name(int64_t m, int64_t n, int64_t k, int64_t lda, int orderA,
                                 int64_t ldb, int orderB, int64_t ldc, int orderC, int a_unsigned,
                                 int b_unsigned, int aligned16) {
  Problem p;
  // stand-in addresses that only carry the alignment
  const void *fake = reinterpret_cast<const void *>(aligned16 ? uintptr_t(4096) : uintptr_t(4097));
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, fake, lda, orderA, fake, ldb,
                                  orderB, reinterpret_cast<int32_t *>(uintptr_t(4096)), ldc,
                                  orderC, MIPGEMM_OVERWRITE, nullptr, 0, &p);
  if (rc != 0) return "invalid";
  return mip::variant_name(mip::choose_variant(p));
}

}  // extern "C"
