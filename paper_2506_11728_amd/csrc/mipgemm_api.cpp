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
    case VARIANT_TILE64X256: return "mfma_tile64x256";
    case VARIANT_TILE256X64: return "mfma_tile256x64";
    default: return "?";
  }
}

// MIPGEMM_VARIANT pins the kernel (tuning and tests): simple, dma256, dma256k128,
// tile256, tile128, tile64, tile64x256, tile256x64.  The two dma variants only apply
// to problems they are eligible for; others keep the automatic choice.
// MIPGEMM_SPLITK pins the number of k ranges of the tile kernels.
static Variant forced_variant() {
  const char *e = std::getenv("MIPGEMM_VARIANT");
  if (!e || !*e) return VARIANT_NONE;
  static const struct { const char *name; Variant v; } table[] = {
      {"simple", VARIANT_SIMPLE},         {"dma256", VARIANT_DMA256},
      {"dma256k128", VARIANT_DMA256K128}, {"tile256", VARIANT_TILE256},
      {"tile128", VARIANT_TILE128},       {"tile64", VARIANT_TILE64},
      {"tile64x256", VARIANT_TILE64X256}, {"tile256x64", VARIANT_TILE256X64}};
  for (const auto &t : table)
    if (!std::strcmp(e, t.name)) return t.v;
  return VARIANT_NONE;
}

static int forced_splits() {
  const char *e = std::getenv("MIPGEMM_SPLITK");
  if (!e || !*e) return 0;
  int v = std::atoi(e);
  return v > 0 ? v : 0;
}

static int64_t tile_count(const Problem &p, int64_t bm, int64_t bn) {
  return ((p.m + bm - 1) / bm) * ((p.n + bn - 1) / bn);
}

static void tile_shape(Variant v, int64_t *bm, int64_t *bn) {
  switch (v) {
    case VARIANT_TILE256: *bm = 256; *bn = 256; break;
    case VARIANT_TILE128: *bm = 128; *bn = 128; break;
    case VARIANT_TILE64X256: *bm = 64; *bn = 256; break;
    case VARIANT_TILE256X64: *bm = 256; *bn = 64; break;
    default: *bm = 64; *bn = 64; break;
  }
}

Plan choose_plan(const Problem &p) {
  constexpr int64_t kComputeUnits = 256;
  if (p.m == 0 || p.n == 0) return {VARIANT_NONE, 1};
  if (p.k == 0) return {p.accumulate ? VARIANT_NONE : VARIANT_FILL, 1};
  Variant v = forced_variant();
  if (v == VARIANT_DMA256 && !dma_eligible(p, false)) v = VARIANT_NONE;
  if (v == VARIANT_DMA256K128 && !dma_eligible(p, true)) v = VARIANT_NONE;
  if (v == VARIANT_NONE) {
    // The largest tile that still gives most compute units a workgroup; a
    // matrix that is short in one dimension takes a tile that is short there too.
    if (tile_count(p, 256, 256) >= 192) {
      // deep k blocks pay off once the k loop is long enough to amortise their prologue
      if (p.k >= 6144 && dma_eligible(p, true)) v = VARIANT_DMA256K128;
      else if (dma_eligible(p, false)) v = VARIANT_DMA256;
      else v = VARIANT_TILE256;
    } else if (p.m <= 64 && p.n > 128) {
      v = VARIANT_TILE64X256;
    } else if (p.n <= 64 && p.m > 128) {
      v = VARIANT_TILE256X64;
    } else if (tile_count(p, 128, 128) >= 192) {
      v = VARIANT_TILE128;
    } else {
      v = VARIANT_TILE64;
    }
  }
  int splits = 1;
  if (v >= VARIANT_TILE256) {
    splits = forced_splits();
    if (splits == 0) {
      // Too few tiles to fill the chip: cut k into ranges, at least 256 deep each,
      // until there are about two workgroups per compute unit.
      int64_t bm, bn;
      tile_shape(v, &bm, &bn);
      const int64_t tiles = tile_count(p, bm, bn);
      const int64_t nkt = (p.k + 63) / 64;
      splits = 1;
      if (tiles < kComputeUnits / 2) {
        int64_t want = (2 * kComputeUnits + tiles - 1) / tiles;
        int64_t most = nkt / 4 > 1 ? nkt / 4 : 1;
        splits = (int)(want < most ? want : most);
      }
    }
  }
  return {v, splits};
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
  const mip::Plan plan = mip::choose_plan(p);
  const mip::Variant v = plan.variant;
  switch (v) {
    case mip::VARIANT_NONE: break;
    case mip::VARIANT_FILL: e = mip::launch_fill_zero(p, s); break;
    case mip::VARIANT_SIMPLE: e = mip::launch_simple(p, s); break;
    case mip::VARIANT_DMA256: e = mip::launch_dma(p, false, s); break;
    case mip::VARIANT_DMA256K128: e = mip::launch_dma(p, true, s); break;
    default: e = mip::launch_tile(p, v, plan.splits, s); break;
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
  return mip::variant_name(mip::choose_plan(p).variant);
}

}  // extern "C"
