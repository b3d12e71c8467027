// C-ABI layer of mipgemm: argument validation, normalisation of the storage
// orders and dispatch to the HIP kernels.  Everything here runs on the host.
#include "../../include/mipgemm.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "mip_internal.h"

namespace mip {

bool dma_eligible(const Problem &p, Shape shape) {
  switch (shape) {
    case SHAPE_256: return dma_eligible_256x256(p);
    case SHAPE_128: return dma_eligible_128x128(p);
    case SHAPE_64: return dma_eligible_64x64(p);
    case SHAPE_64X256: return dma_eligible_64x256(p);
    case SHAPE_256X64: return dma_eligible_256x64(p);
    case SHAPE_64X128: return dma_eligible_64x128(p);
    case SHAPE_128X64: return dma_eligible_128x64(p);
    default: return false;
  }
}

hipError_t launch_dma(const Problem &p, Shape shape, int splits, hipStream_t s) {
  switch (shape) {
    case SHAPE_256: return launch_dma_256x256(p, splits, s);
    case SHAPE_128: return launch_dma_128x128(p, splits, s);
    case SHAPE_64: return launch_dma_64x64(p, splits, s);
    case SHAPE_64X256: return launch_dma_64x256(p, splits, s);
    case SHAPE_256X64: return launch_dma_256x64(p, splits, s);
    case SHAPE_64X128: return launch_dma_64x128(p, splits, s);
    case SHAPE_128X64: return launch_dma_128x64(p, splits, s);
    default: return hipErrorInvalidValue;
  }
}

static const char *const kShapeNames[SHAPE_COUNT] = {"256", "128", "64", "64x256", "256x64",
                                                     "64x128", "128x64"};
static const int64_t kShapeRows[SHAPE_COUNT] = {256, 128, 64, 64, 256, 64, 128};
static const int64_t kShapeCols[SHAPE_COUNT] = {256, 128, 64, 256, 64, 128, 64};

const char *plan_name(const Plan &plan) {
  static const char *const staged[SHAPE_COUNT] = {"mfma_tile256", "mfma_tile128", "mfma_tile64",
                                                  "mfma_tile64x256", "mfma_tile256x64",
                                                  "mfma_tile64x128", "mfma_tile128x64"};
  static const char *const dma[SHAPE_COUNT] = {"mfma_dma256", "mfma_dma128", "mfma_dma64",
                                               "mfma_dma64x256", "mfma_dma256x64",
                                               "mfma_dma64x128", "mfma_dma128x64"};
  switch (plan.kind) {
    case KIND_NONE: return "none";
    case KIND_FILL: return "fill_zero";
    case KIND_SIMPLE: return "simple";
    case KIND_STAGED: return staged[plan.shape];
    case KIND_DMA: return dma[plan.shape];
    case KIND_DMA_K128: return "mfma_dma256_k128";
    case KIND_SLAB: return plan.splits == 2 ? "mfma_slab32" : "mfma_slab16";
    default: return "?";
  }
}

// MIPGEMM_VARIANT pins the kernel (tuning and tests): "simple", "dma256k128",
// "slab16" / "slab32" (the skinny-m kernel with that slab width),
// "tile<shape>" (register-staged) or "dma<shape>" (direct-to-LDS) with <shape> one of
// 256, 128, 64, 64x256, 256x64, 64x128, 128x64.  A dma variant only applies to problems it is
// eligible for; others fall back to the staged kernel of the same shape.
// MIPGEMM_SPLITK pins the number of k ranges of the tile kernels.
static bool forced_plan(const Problem &p, Plan *plan) {
  const char *e = std::getenv("MIPGEMM_VARIANT");
  if (!e || !*e) return false;
  if (!std::strcmp(e, "simple")) { *plan = {KIND_SIMPLE, SHAPE_64, 1}; return true; }
  if (!std::strcmp(e, "dma256k128")) {
    if (!dma_k128_eligible(p)) return false;
    *plan = {KIND_DMA_K128, SHAPE_256, 1};
    return true;
  }
  if (!std::strcmp(e, "slab16") || !std::strcmp(e, "slab32")) {
    const int nt = e[4] == '3' ? 2 : 1;
    if (!slab_eligible(p, nt)) return false;
    *plan = {KIND_SLAB, SHAPE_64, nt};
    return true;
  }
  const bool want_dma = !std::strncmp(e, "dma", 3);
  if (!want_dma && std::strncmp(e, "tile", 4)) return false;
  const char *shape = e + (want_dma ? 3 : 4);
  for (int i = 0; i < SHAPE_COUNT; ++i)
    if (!std::strcmp(shape, kShapeNames[i])) {
      const Shape sh = static_cast<Shape>(i);
      *plan = {want_dma && dma_eligible(p, sh) ? KIND_DMA : KIND_STAGED, sh, 1};
      return true;
    }
  return false;
}

static int forced_splits() {
  const char *e = std::getenv("MIPGEMM_SPLITK");
  if (!e || !*e) return 0;
  int v = std::atoi(e);
  return v > 0 ? v : 0;
}

// over all problems of a batch: what the chip sees is their sum
static int64_t tile_count(const Problem &p, Shape s) {
  return ((p.m + kShapeRows[s] - 1) / kShapeRows[s]) * ((p.n + kShapeCols[s] - 1) / kShapeCols[s]) *
         (p.batch > 1 ? p.batch : 1);
}

Plan choose_plan(const Problem &p) {
  constexpr int64_t kComputeUnits = 256;
  if (p.m == 0 || p.n == 0) return {KIND_NONE, SHAPE_64, 1};
  if (p.k == 0) return {p.accumulate ? KIND_NONE : KIND_FILL, SHAPE_64, 1};
  Plan plan;
  if (!forced_plan(p, &plan)) {
    // The largest tile that still gives most compute units a workgroup; a
    // matrix that is short in one dimension takes a tile that is short there too.
    // A short side (a few tokens, a few output channels) makes the problem a
    // stream over the long operand: wide tiles only when the long side alone
    // fills the chip, else 64 x 64 tiles, which give four times as many workgroups.
    // With at most 16 rows the atomics of split k are cheap, and wide tiles (whole
    // cache lines of a row-major operand) win as soon as k is long enough to cut
    // into one range of 8 blocks or more per compute unit.
    Shape sh;
    const int64_t ranges = p.k / 512 > 1 ? p.k / 512 : 1;
    auto enough = [&](Shape wide, int64_t short_side) {
      const int64_t t = tile_count(p, wide);
      return t >= kComputeUnits || (short_side <= 16 && !p.out_float && t * ranges >= kComputeUnits);
    };
    if (p.m <= 64 && p.n > 128) sh = enough(SHAPE_64X256, p.m) ? SHAPE_64X256 : SHAPE_64;
    else if (p.n <= 64 && p.m > 128) sh = enough(SHAPE_256X64, p.n) ? SHAPE_256X64 : SHAPE_64;
    // A large tile buys operand reuse, which only a long k turns into time: with a short
    // k the problem is a stream that ends in the write of C, and small tiles, several
    // workgroups to a compute unit, overlap that write with the next tile's loads.
    // Between 128 x 128 (too few tiles) and 64 x 64 (64 operations per operand byte,
    // which the L2 caches cannot feed) sit the 8192-element tiles, long side along the
    // longer dimension of C.
    else if (p.k >= 1024 && tile_count(p, SHAPE_256) >= 192) sh = SHAPE_256;
    else if (p.k >= 512 && tile_count(p, SHAPE_128) >= kComputeUnits) sh = SHAPE_128;
    else if (p.k >= 512 && tile_count(p, p.m >= p.n ? SHAPE_128X64 : SHAPE_64X128) >= kComputeUnits &&
             dma_eligible(p, p.m >= p.n ? SHAPE_128X64 : SHAPE_64X128))
      sh = p.m >= p.n ? SHAPE_128X64 : SHAPE_64X128;  // (measured on the direct-to-LDS kernels only)
    else if (p.k >= 512 && tile_count(p, SHAPE_128) >= 192) sh = SHAPE_128;
    else sh = SHAPE_64;
    // deep k blocks pay off once the k loop is long enough to amortise their prologue
    // A few rows of A against a k-contiguous B is one pass over B with nothing to
    // share: a workgroup per 16-column slab does it in one launch, without atomics.
    // (A row-major B would reach each slab in 16-byte pieces of its cache lines,
    // which the tiled kernels, with their 64-byte pieces and split k, do better.)
    // The same kernel serves short k, where the tiled kernels cannot split k
    // and 64-column tiles leave most compute units idle.
    const bool slab_ok = p.m <= 64 && slab_eligible(p, 1);
    if (slab_ok && p.b_sk == 1 && p.m <= 16 && p.n / 16 >= 192) plan = {KIND_SLAB, SHAPE_64, 1};
    else if (slab_ok && p.k < 1024 && tile_count(p, SHAPE_64) < kComputeUnits / 2 && p.n / 16 >= 64)
      plan = {KIND_SLAB, SHAPE_64, 1};
    else if (sh == SHAPE_256 && p.k >= 2048 && dma_k128_eligible(p)) plan = {KIND_DMA_K128, sh, 1};
    else if (dma_eligible(p, sh)) plan = {KIND_DMA, sh, 1};
    // the register-staged kernel keeps its operands in flight in VGPRs, which a
    // 256 x 256 tile's accumulators leave no room for: it runs faster on 128 x 128
    else plan = {KIND_STAGED, sh == SHAPE_256 ? SHAPE_128 : sh, 1};
  }
  if (plan.kind == KIND_STAGED || plan.kind == KIND_DMA) {
    plan.splits = p.out_float ? 1 : forced_splits();  // float sums are not combined out of order
    if (plan.splits == 0) {
      // Too few tiles to fill the chip: cut k into ranges of at least 512 (128 for the
      // register-staged kernel) until
      // there is about one workgroup per compute unit.  Every range adds its
      // partial sums into C with atomics (and an overwrite needs C zeroed first),
      // so short problems (few rows of C per byte of operand) may split further
      // than tall ones.
      const int64_t tiles = tile_count(p, plan.shape);
      const int64_t nkt = (p.k + 63) / 64;
      plan.splits = 1;
      // a stream over one long operand (short side of a few rows) is bound by memory
      // latency: it wants two workgroups per compute unit in flight
      const int64_t short_side = p.m < p.n ? p.m : p.n;
      // (of the 64 x 64 tiles, that is: the wide ones fill a compute unit's LDS alone,
      // and one workgroup too many would cost a second round)
      const bool small_tile = plan.shape == SHAPE_64;
      const int64_t target = short_side <= 16 && small_tile ? 2 * kComputeUnits : kComputeUnits;
      if (tiles < target / 2 && !p.out_float) {
        const int64_t want = short_side <= 16 && small_tile ? (target + tiles - 1) / tiles : target / tiles;
        // the register-staged kernel has a shallow pipeline with little to amortise:
        // ranges of two k blocks already pay, and it tolerates twice the atomics
        const bool staged = plan.kind == KIND_STAGED;
        const int64_t shortest = staged ? 2 : 8;  // k blocks per range
        const int64_t most = nkt / shortest > 1 ? nkt / shortest : 1;
        const int64_t atomics_ok = (short_side <= 16 ? 64 : (short_side <= 64 ? 8 : 4)) * (staged ? 2 : 1);
        int64_t sp = want < most ? want : most;
        if (sp > atomics_ok) sp = atomics_ok;
        plan.splits = (int)sp;
      }
    }
  }
  return plan;
}

}  // namespace mip

namespace {

using mip::Problem;

bool order_ok(int o) { return o == MIPGEMM_ROW_MAJOR || o == MIPGEMM_COL_MAJOR; }

// Fills `out` and returns 0, or returns the negative argument number.
int validate_and_normalise(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k,
                           const void *A, int64_t lda, int orderA, const void *B, int64_t ldb,
                           int orderB, void *C, int64_t ldc, int orderC, int mode,
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
  p.C = static_cast<int32_t *>(C);
  p.ldc = ldc;
  p.accumulate = mode == MIPGEMM_ACCUMULATE;
  p.out_float = 0;
  p.scale = 1.0f;
  *out = p;
  return 0;
}

struct Batch {
  int64_t count = 1;
  int64_t stride_a = 0, stride_b = 0, stride_c = 0;  // elements between consecutive problems
};

// out_float: C holds floats and receives float(sum) * scale (the f32 entry points)
int run(int a_unsigned, int b_unsigned, int out_float, float scale, int64_t m, int64_t n,
        int64_t k, const void *A, int64_t lda, int orderA, const void *B, int64_t ldb, int orderB,
        void *C, int64_t ldc, int orderC, int mode, void *workspace, size_t workspace_bytes,
        void *stream, const Batch &batch = Batch()) {
  Problem p;
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB,
                                  C, ldc, orderC, mode, workspace, workspace_bytes, &p);
  if (rc != 0) return rc;
  p.out_float = out_float;
  p.scale = scale;
  p.batch = batch.count;
  // a column-major C has swapped the operand roles: the strides follow their operands
  const bool swapped = orderC != MIPGEMM_ROW_MAJOR;
  p.a_sb = swapped ? batch.stride_b : batch.stride_a;
  p.b_sb = swapped ? batch.stride_a : batch.stride_b;
  p.c_sb = batch.stride_c;
  if (p.batch == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  const mip::Plan plan = mip::choose_plan(p);
  switch (plan.kind) {
    case mip::KIND_NONE: break;
    case mip::KIND_FILL: e = mip::launch_fill_zero(p, s); break;
    case mip::KIND_SIMPLE: e = mip::launch_simple(p, s); break;
    case mip::KIND_STAGED: e = mip::launch_staged(p, plan.shape, plan.splits, s); break;
    case mip::KIND_DMA: e = mip::launch_dma(p, plan.shape, plan.splits, s); break;
    case mip::KIND_DMA_K128: e = mip::launch_dma_k128(p, s); break;
    case mip::KIND_SLAB: e = mip::launch_slab(p, plan.splits, s); break;
  }
  return static_cast<int>(e);
}

}  // namespace

extern "C" {

int mipgemm_s8s8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(0, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_u8s8s32(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(1, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_s8u8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return run(0, 1, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_s8s8s32_batched(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda,
                            int orderA, int64_t strideA, const int8_t *B, int64_t ldb, int orderB,
                            int64_t strideB, int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode, void *workspace, size_t workspace_bytes,
                            void *stream) {
  // the shared validation numbers its arguments as the single-problem entry points do:
  // map them onto this prototype (strides and batch shift everything after orderA)
  static const int renumber[17] = {0, 1, 2, 3, 4, 5, 6, 8, 9, 10, 12, 13, 14, 17, 18, 19, 20};
  Problem probe;
  const int base = validate_and_normalise(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
                                          orderC, mode, workspace, workspace_bytes, &probe);
  int first_bad = base < 0 ? renumber[-base] : 0;  // the lowest-numbered invalid argument wins
  auto also = [&](int number, bool bad) {
    if (bad && (first_bad == 0 || number < first_bad)) first_bad = number;
  };
  also(7, strideA < 0);
  also(11, strideB < 0);
  also(15, strideC < 0);
  also(16, batch < 0 || batch > 65535);
  if (first_bad) return -first_bad;
  Batch b;
  b.count = batch;
  b.stride_a = strideA;
  b.stride_b = strideB;
  b.stride_c = strideC;
  return run(0, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
             workspace, workspace_bytes, stream, b);
}

// Dequantised output (paper Section 7.3).  Same arguments and numbering as the
// s32 entry points; scale is argument 17.
static int run_f32(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k, const void *A,
                   int64_t lda, int orderA, const void *B, int64_t ldb, int orderB, float *C,
                   int64_t ldc, int orderC, int mode, void *workspace, size_t workspace_bytes,
                   void *stream, float scale) {
  if (!(scale == scale) || scale - scale != 0.0f) {  // NaN or infinity
    // still report an earlier invalid argument first
    Problem p;
    int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb,
                                    orderB, C, ldc, orderC, mode, workspace, workspace_bytes, &p);
    return rc != 0 ? rc : -17;
  }
  return run(a_unsigned, b_unsigned, 1, scale, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
             orderC, mode, workspace, workspace_bytes, stream);
}

int mipgemm_s8s8f32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, float *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_f32(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                 workspace_bytes, stream, scale);
}

int mipgemm_u8s8f32(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, float *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_f32(1, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                 workspace_bytes, stream, scale);
}

int mipgemm_s8u8f32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB, float *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_f32(0, 1, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                 workspace_bytes, stream, scale);
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
      "invalid argument 15 (workspace_bytes too small)", "invalid argument 16 (stream)",
      "invalid argument 17 (scale is not finite)", "invalid argument 18", "invalid argument 19",
      "invalid argument 20"};
  if (code <= 0 && code >= -20) return args[-code];
  if (code > 0) return hipGetErrorString(static_cast<hipError_t>(code));
  return "unknown mipgemm error code";
}

}  // extern "C"

// ---------------------------------------------------------------------------
// convolution by lowering (paper Section 7.2)
// ---------------------------------------------------------------------------
namespace {

struct ConvCall {
  mip::ConvGeom geom;
  int64_t rows;  // b * h_o * w_o: the GEMM's n
  int64_t k;     // h_f * w_f * c_i
  int64_t ldm;   // row pitch of a written-out augmented matrix
};

// 0 and `out`, or the negative number of the first bad size argument; `co_arg` < 0 for
// the entry point that has no c_o (then hf .. pad are arguments 5 .. 8 instead of 6 .. 9)
int conv_sizes(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co, bool has_co, int64_t hf,
               int64_t wf, int64_t stride, int64_t pad, ConvCall *out) {
  const int64_t lim = (int64_t)1 << 31;
  const int shift = has_co ? 1 : 0;
  if (b < 0 || b >= lim) return -1;
  if (hi < 1 || hi >= lim) return -2;
  if (wi < 1 || wi >= lim) return -3;
  if (ci < 1 || ci >= lim) return -4;
  if (has_co && (co < 0 || co >= lim)) return -5;
  if (hf < 1 || hf >= lim) return -(5 + shift);
  if (wf < 1 || wf >= lim) return -(6 + shift);
  if (stride < 1 || stride >= lim) return -(7 + shift);
  if (pad < 0 || pad >= lim) return -(8 + shift);
  if (hf > hi + 2 * pad) return -(5 + shift);  // the filter must fit the padded image
  if (wf > wi + 2 * pad) return -(6 + shift);
  const int64_t ho = (hi + 2 * pad - hf) / stride + 1, wo = (wi + 2 * pad - wf) / stride + 1;
  // products checked step by step so that none overflows 64 bits
  if (hi * wi >= lim || hi * wi * ci >= lim || (b > 0 && hi * wi * ci >= lim / b)) return -1;
  if (ho >= lim || wo >= lim) return -(8 + shift);  // only an absurd padding gets here
  if (ho * wo >= lim || (b > 0 && ho * wo >= lim / b)) return -1;
  if (hf * wf >= lim || hf * wf * ci >= lim) return -4;
  out->geom = mip::ConvGeom{(int)hi, (int)wi, (int)ci, (int)wf, (int)ho, (int)wo, (int)stride, (int)pad};
  out->rows = b * ho * wo;
  out->k = hf * wf * ci;
  out->ldm = (out->k + 15) / 16 * 16;
  return 0;
}

// the GEMM the convolution is lowered to, in the kernels' terms: the row-major C is O
// seen as (b h_o w_o) x c_o, its A the augmented matrix, its B the filters (k contiguous)
Problem conv_problem(const ConvCall &c, int64_t co, const void *F, const void *I, void *O, int mode,
                     bool implicit, const void *M, int out_float = 0, float scale = 1.0f) {
  Problem p;
  p.m = c.rows; p.n = co; p.k = c.k;
  p.A = implicit ? I : M; p.a_sm = implicit ? c.k : c.ldm; p.a_sk = 1; p.a_unsigned = 1;
  p.B = F; p.b_sk = 1; p.b_sn = c.k; p.b_unsigned = 0;
  p.C = static_cast<int32_t *>(O); p.ldc = co;
  p.accumulate = mode == MIPGEMM_ACCUMULATE;
  p.out_float = out_float; p.scale = scale;
  p.conv = nullptr;
  return p;
}

// whether the gathering kernel serves this convolution, and with which plan
bool conv_implicit_plan(const ConvCall &c, Problem p, mip::Plan *plan) {
  const char *e = std::getenv("MIPGEMM_CONV");  // "im2col" pins the written-out path (tests, tuning)
  if (e && !std::strcmp(e, "im2col")) return false;
  if (p.m == 0 || p.n == 0) return false;
  p.conv = &c.geom;
  *plan = mip::choose_plan(p);
  return plan->kind == mip::KIND_DMA;
}

}  // namespace

extern "C" {

size_t mipgemm_conv_workspace_size(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                   int64_t hf, int64_t wf, int64_t stride, int64_t pad) {
  ConvCall c;
  if (conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c) != 0) return 0;
  if (c.rows == 0 || co == 0) return 0;
  const void *fake = reinterpret_cast<const void *>(uintptr_t(4096));
  mip::Plan plan;
  if (conv_implicit_plan(c, conv_problem(c, co, fake, fake, const_cast<void *>(fake),
                                         MIPGEMM_OVERWRITE, true, nullptr), &plan))
    return 0;
  return static_cast<size_t>(c.rows) * static_cast<size_t>(c.ldm);
}

const char *mipgemm_conv_variant_name(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                      int64_t hf, int64_t wf, int64_t stride, int64_t pad) {
  ConvCall c;
  if (conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c) != 0) return "invalid";
  if (c.rows == 0 || co == 0) return "none";
  const void *fake = reinterpret_cast<const void *>(uintptr_t(4096));
  mip::Plan plan;
  const bool implicit = conv_implicit_plan(
      c, conv_problem(c, co, fake, fake, const_cast<void *>(fake), MIPGEMM_OVERWRITE, true, nullptr),
      &plan);
  if (!implicit)
    plan = mip::choose_plan(conv_problem(c, co, fake, fake, const_cast<void *>(fake),
                                         MIPGEMM_OVERWRITE, false, fake));
  // static strings: every kernel variant name with either prefix
#define MIP_NAME(x) {x, "implicit:" x, "im2col+" x}
  static const char *const names[][3] = {
      MIP_NAME("mfma_dma256"), MIP_NAME("mfma_dma128"), MIP_NAME("mfma_dma64"),
      MIP_NAME("mfma_dma64x256"), MIP_NAME("mfma_dma256x64"), MIP_NAME("mfma_tile256"),
      MIP_NAME("mfma_tile128"), MIP_NAME("mfma_tile64"), MIP_NAME("mfma_tile64x256"),
      MIP_NAME("mfma_tile256x64"), MIP_NAME("mfma_dma64x128"), MIP_NAME("mfma_dma128x64"),
      MIP_NAME("mfma_tile64x128"), MIP_NAME("mfma_tile128x64"), MIP_NAME("mfma_dma256_k128"), MIP_NAME("mfma_slab16"),
      MIP_NAME("mfma_slab32"), MIP_NAME("simple")};
#undef MIP_NAME
  const char *base = mip::plan_name(plan);
  for (const auto &n : names)
    if (!std::strcmp(n[0], base)) return n[implicit ? 1 : 2];
  return implicit ? "implicit" : "im2col";
}

int mipgemm_im2col_u8(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t hf, int64_t wf,
                      int64_t stride, int64_t pad, const uint8_t *I, uint8_t *M, int64_t ldm,
                      void *stream) {
  ConvCall c;
  int rc = conv_sizes(b, hi, wi, ci, 0, false, hf, wf, stride, pad, &c);
  if (rc != 0) return rc;
  if (!I && b > 0) return -9;
  if (!M && c.rows > 0) return -10;
  if (ldm < c.k || ldm > MIPGEMM_MAX_DIM) return -11;
  return static_cast<int>(mip::launch_im2col(c.geom, c.rows, c.k, I, M, ldm,
                                             static_cast<hipStream_t>(stream)));
}

static int run_conv(int out_float, float scale, int64_t b, int64_t hi, int64_t wi, int64_t ci,
                    int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad, const int8_t *F,
                    const uint8_t *I, void *O, int mode, void *workspace, size_t workspace_bytes,
                    void *stream) {
  ConvCall c;
  int rc = conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c);
  if (rc != 0) return rc;
  if (!F && co > 0) return -10;
  if (!I && b > 0) return -11;
  if (!O && c.rows > 0 && co > 0) return -12;
  if (mode != MIPGEMM_OVERWRITE && mode != MIPGEMM_ACCUMULATE) return -13;
  if (out_float && (!(scale == scale) || scale - scale != 0.0f)) return -17;  // NaN or infinity
  if (c.rows == 0 || co == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  mip::Plan plan;
  Problem p = conv_problem(c, co, F, I, O, mode, true, nullptr, out_float, scale);
  if (conv_implicit_plan(c, p, &plan)) {
    p.conv = &c.geom;
    return static_cast<int>(mip::launch_dma(p, plan.shape, plan.splits, s));
  }
  const size_t need = static_cast<size_t>(c.rows) * static_cast<size_t>(c.ldm);
  if (!workspace) return -14;
  if (workspace_bytes < need) return -15;
  hipError_t e = mip::launch_im2col(c.geom, c.rows, c.k, I, static_cast<uint8_t *>(workspace), c.ldm, s);
  if (e != hipSuccess) return static_cast<int>(e);
  // F is A (c_o x k, row-major), the matrix just written is B (k x n, column-major),
  // O is C (column-major, ldc = c_o)
  return run(0, 1, out_float, scale, co, c.rows, c.k, F, c.k, MIPGEMM_ROW_MAJOR, workspace, c.ldm,
             MIPGEMM_COL_MAJOR, O, co, MIPGEMM_COL_MAJOR, mode, nullptr, 0, stream);
}

int mipgemm_conv_s8u8s32(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co, int64_t hf,
                         int64_t wf, int64_t stride, int64_t pad, const int8_t *F, const uint8_t *I,
                         int32_t *O, int mode, void *workspace, size_t workspace_bytes,
                         void *stream) {
  return run_conv(0, 1.0f, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream);
}

int mipgemm_conv_s8u8f32(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co, int64_t hf,
                         int64_t wf, int64_t stride, int64_t pad, const int8_t *F, const uint8_t *I,
                         float *O, int mode, void *workspace, size_t workspace_bytes, void *stream,
                         float scale) {
  return run_conv(1, scale, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream);
}

int mipgemm_pack_b(int64_t k, int64_t n, const void *B, int64_t ldb, int orderB, void *P,
                   int64_t ldp, void *stream) {
  if (k < 0 || k > MIPGEMM_MAX_DIM) return -1;
  if (n < 0 || n > MIPGEMM_MAX_DIM) return -2;
  if (!B && k > 0 && n > 0) return -3;
  if (!order_ok(orderB)) return -5;
  {
    const int64_t need = orderB == MIPGEMM_ROW_MAJOR ? n : k;
    if (ldb < (need > 1 ? need : 1) || ldb > MIPGEMM_MAX_DIM) return -4;
  }
  if (!P && k > 0 && n > 0) return -6;
  if (ldp < (k > 1 ? k : 1) || ldp > MIPGEMM_MAX_DIM) return -7;
  return static_cast<int>(mip::launch_pack_b(k, n, static_cast<const uint8_t *>(B), ldb,
                                             orderB == MIPGEMM_COL_MAJOR, static_cast<uint8_t *>(P),
                                             ldp, static_cast<hipStream_t>(stream)));
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
  return mip::plan_name(mip::choose_plan(p));
}

}  // extern "C"
