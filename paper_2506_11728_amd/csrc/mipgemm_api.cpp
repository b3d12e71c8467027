// C-ABI layer of mipgemm, GEMM entry points: argument validation, normalisation of the
// storage orders and hand-over to the dispatcher.  Everything here runs on the host.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "api_internal.h"
#include "tuning.h"

namespace mip {

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
  if (workspace_bytes > 0 && !workspace) return -14;  // the workspace itself is optional

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

// The packed route: operands that the direct-to-LDS kernels cannot stream (a base or a
// leading dimension that is not a multiple of 16 bytes, k not a multiple of 64) are first
// rewritten into the workspace.  Worth two more launches and one more pass over A and B once
// the product is big enough and neither side is skinny.
static int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }
// long k: a multiple of 128 for the kernel with 128-deep k blocks; short k: of 64
static int64_t padded_k(int64_t k) { return k >= 1024 ? round_up(k, 128) : round_up(k, 64); }
// rows in whole tiles of 256, so that the kernel for large problems may fetch whole tiles
static size_t packed_bytes(int64_t m, int64_t n, int64_t k) {
  return static_cast<size_t>((round_up(m, 256) + round_up(n, 256)) * padded_k(k));
}
// sizes whose packed operands would not fit 2^62 bytes are never packed: no overflow in the sums
static bool packable(int64_t m, int64_t n, int64_t k) {
  return ((double)m + (double)n + 512.0) * ((double)k + 128.0) < 4.0e18;
}
static bool packing_size_ok(int64_t m, int64_t n, int64_t k) {
  if (!packable(m, n, k)) return false;
  // measured (us, worst to best layout, in place -> packed): 200^3 8.4-7.7 -> 7.5-7.3,
  // 800^3 19-11 -> 9.8-9.4, 100 x 100 x 10001 35-18 -> 15, 128 x 3001 x 513 12.6-10.3 -> 9.6-8.8;
  // but 64 x 1000 x 1000 8.8-7.8 -> 10, 1000^2 x 100 7.8-6.6 -> 8.3, 16 x 11009 x 4099 38-28 -> 45-31
  return m >= 96 && n >= 96 && k >= 192 && (double)m * (double)n * (double)k >= 4194304.0;  // 2^22
}
// The tuning value MIPGEMM_PACK pins the decision for tests and tuning: "always" packs whatever the
// direct-to-LDS kernels cannot stream, however small; "never" leaves everything in place.
static bool packing_pays(const Problem &p, const mip::Plan &plan) {
  if (plan.kind != mip::KIND_STAGED && plan.kind != mip::KIND_SIMPLE) return false;
  if (p.batch != 1 || p.conv || p.m < 1 || p.n < 1 || p.k < 1 || !packable(p.m, p.n, p.k)) return false;
  if (tuning().pack > 0) return true;
  if (tuning().pack < 0) return false;
  return packing_size_ok(p.m, p.n, p.k);
}

size_t packed_route_bytes(const Problem &p) {
  return packing_pays(p, choose_plan(p)) ? packed_bytes(p.m, p.n, p.k) : 0;
}

int run_gemm(int a_unsigned, int b_unsigned, int out_float, float scale, int64_t m, int64_t n,
        int64_t k, const void *A, int64_t lda, int orderA, const void *B, int64_t ldb, int orderB,
        void *C, int64_t ldc, int orderC, int mode, void *workspace, size_t workspace_bytes,
        void *stream, const Batch &batch, const int32_t *ksum) {
  Problem p;
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB,
                                  C, ldc, orderC, mode, workspace, workspace_bytes, &p);
  if (rc != 0) return rc;
  // (the sums belong to the signed operand whichever role the normalisation has given it)
  p.ksum = (a_unsigned != 0) != (b_unsigned != 0) ? ksum : nullptr;
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
  // what the kernels may use of the workspace: all of it, or what the packed operands leave
  uint8_t *ws = static_cast<uint8_t *>(workspace);
  size_t ws_bytes = workspace ? workspace_bytes : 0;
  if (reinterpret_cast<uintptr_t>(ws) % 16 != 0 && ws_bytes > 0) {  // slots are read 16 bytes at a time
    const size_t skip = 16 - reinterpret_cast<uintptr_t>(ws) % 16;
    ws = skip < ws_bytes ? ws + skip : nullptr;
    ws_bytes = skip < ws_bytes ? ws_bytes - skip : 0;
  }
  p.ws = ws_bytes ? ws : nullptr;
  p.ws_bytes = ws_bytes;
  mip::Plan plan = mip::choose_plan(p);
  if (packing_pays(p, plan) && workspace && workspace_bytes >= packed_bytes(p.m, p.n, p.k)) {
    // Pack A and Pack B (paper Section 4.1) into aligned, k-contiguous buffers with the k
    // tail zeroed, so that the direct-to-LDS kernels can stream them
    const int64_t kp = padded_k(p.k);
    uint8_t *Ap = static_cast<uint8_t *>(workspace);
    uint8_t *Bp = Ap + round_up(p.m, 256) * kp;
    e = mip::launch_pack_pair(p.k, kp, p.m, static_cast<const uint8_t *>(p.A),
                              p.a_sk == 1 ? p.a_sm : p.a_sk, p.a_sk == 1, Ap, p.n,
                              static_cast<const uint8_t *>(p.B), p.b_sk == 1 ? p.b_sn : p.b_sk,
                              p.b_sk == 1, Bp, kp, s);
    if (e != hipSuccess) return static_cast<int>(e);
    p.A = Ap; p.a_sm = kp; p.a_sk = 1;
    p.B = Bp; p.b_sn = kp; p.b_sk = 1;
    p.k = kp;
    p.rows_padded_to_256 = true;
    // the packed operands keep the front of the workspace
    const size_t used = (packed_bytes(p.m, p.n, kp) + 255) / 256 * 256;
    p.ws = workspace_bytes > used ? static_cast<uint8_t *>(workspace) + used : nullptr;
    p.ws_bytes = workspace_bytes > used ? workspace_bytes - used : 0;
    if (p.ws && reinterpret_cast<uintptr_t>(p.ws) % 16 != 0) { p.ws = nullptr; p.ws_bytes = 0; }
    plan = mip::choose_plan(p);
  }
  return static_cast<int>(launch_plan(p, plan, s));
}

hipError_t launch_plan(const Problem &p, const Plan &plan, hipStream_t s) {
  switch (plan.kind) {
    case KIND_NONE: return hipSuccess;
    case KIND_FILL: return launch_fill_zero(p, s);
    case KIND_SIMPLE: return launch_simple(p, s);
    case KIND_STAGED: return launch_staged(p, plan.shape, plan.splits, s);
    case KIND_DMA: return launch_dma(p, plan.shape, plan.splits, s);
    case KIND_DMA_K128: return launch_dma_k128(p, s, nullptr, plan.shape == SHAPE_128);
    case KIND_DMA_K128_SPLIT: return launch_dma_k128_split(p, plan.splits, s, plan.shape == SHAPE_256);
    case KIND_SLAB: return launch_slab(p, plan.splits, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace mip

using mip::Batch;
using mip::Problem;
using mip::validate_and_normalise;

extern "C" {

int mipgemm_s8s8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return mip::run_gemm(0, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

int mipgemm_s8s8s32_clocked(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda,
                            int orderA, const int8_t *B, int64_t ldb, int orderB, int32_t *C,
                            int64_t ldc, int orderC, int mode, void *stream,
                            unsigned long long *clocks, size_t clocks_bytes) {
  Problem p;
  int rc = validate_and_normalise(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                                  nullptr, 0, &p);
  if (rc != 0) return rc;
  if (!clocks) return -15;
  if (p.m == 0 || p.n == 0 || p.k == 0 || !mip::dma_k128_eligible(p)) return -1;
  const size_t tiles = static_cast<size_t>(((p.m + 255) / 256) * ((p.n + 255) / 256));
  if (clocks_bytes < (tiles + 7) / 8 * 8 * 2 * sizeof(unsigned long long)) return -16;
  return static_cast<int>(mip::launch_dma_k128(p, static_cast<hipStream_t>(stream), clocks));
}

int mipgemm_u8s8s32(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return mip::run_gemm(1, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

// ---- pre-packed weights ----

static int64_t round_up_to(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

// Layout of the packed weights: columns k-contiguous with pitch kp (k rounded up to whole k
// blocks: 128 bytes from k = 1024 on, 64 below, at least one block), `cols` columns (n rounded
// up to a multiple of 256, at least 256; the added ones zero), then n int32 k-sums.
struct PackedLayout { int64_t kp, cols; size_t sums_at, total; };
static bool packed_layout(int64_t k, int64_t n, PackedLayout *L) {
  if (k < 0 || n < 0 || k > MIPGEMM_MAX_DIM || n > MIPGEMM_MAX_DIM) return false;
  const int64_t block = k >= 1024 ? 128 : 64;
  L->kp = k > 0 ? round_up_to(k, block) : block;
  L->cols = n > 0 ? round_up_to(n, 256) : 256;
  if (L->kp > MIPGEMM_MAX_DIM || (double)L->kp * (double)L->cols > 4.0e18) return false;
  L->sums_at = (size_t)L->kp * (size_t)L->cols;
  L->total = L->sums_at + 4 * (size_t)n;
  return true;
}

size_t mipgemm_packed_weights_bytes(int64_t k, int64_t n) {
  PackedLayout L;
  return packed_layout(k, n, &L) ? L.total : 0;
}

int mipgemm_pack_weights(int64_t k, int64_t n, const int8_t *B, int64_t ldb, int orderB,
                         void *packed, size_t packed_bytes, void *stream) {
  PackedLayout L;
  if (k < 0 || k > MIPGEMM_MAX_DIM) return -1;
  if (n < 0 || n > MIPGEMM_MAX_DIM) return -2;
  if (!B && k > 0 && n > 0) return -3;
  if (!mip::order_ok(orderB)) return -5;
  {
    const int64_t need = orderB == MIPGEMM_ROW_MAJOR ? n : k;
    if (ldb < (need > 1 ? need : 1) || ldb > MIPGEMM_MAX_DIM) return -4;
  }
  if (!packed || reinterpret_cast<uintptr_t>(packed) % 16 != 0) return -6;
  if (!packed_layout(k, n, &L) || packed_bytes < L.total) return -7;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t *body = static_cast<uint8_t *>(packed);
  // the columns, each with its k tail zeroed up to the pitch
  hipError_t e = mip::launch_pack_b(k, n, reinterpret_cast<const uint8_t *>(B), ldb,
                                    orderB == MIPGEMM_COL_MAJOR, body, L.kp, s, L.kp);
  if (e != hipSuccess) return static_cast<int>(e);
  if (k == 0 && n > 0) {  // nothing was moved: the one block of every column is all padding
    mip::Problem z;
    z.m = n; z.n = L.kp / 4; z.k = 0;  // one row of words per column
    z.C = reinterpret_cast<int32_t *>(body); z.ldc = z.n;
    e = mip::launch_fill_zero(z, s);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  if (L.cols > n) {  // the added columns (a fill kernel, not a memset: the call may be under graph capture)
    mip::Problem z;
    z.m = L.cols - n; z.n = L.kp / 4; z.k = 0;  // one row of words per column
    z.C = reinterpret_cast<int32_t *>(body + (size_t)n * (size_t)L.kp); z.ldc = z.n;
    e = mip::launch_fill_zero(z, s);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  e = mip::launch_column_sums(L.kp, n, body, L.kp, reinterpret_cast<int32_t *>(body + L.sums_at), s);
  return static_cast<int>(e);
}

// The GEMM on packed weights: they are B, column-major with the pitch of the layout, and
// bring the k sums an unsigned A needs.  Error numbers follow this prototype (m=1 n=2 k=3 A=4
// lda=5 orderA=6 packed=7 C=8 ldc=9 orderC=10 mode=11 workspace=12).
static int run_packed(int a_unsigned, int64_t m, int64_t n, int64_t k, const void *A, int64_t lda,
                      int orderA, const void *packed, void *C, int64_t ldc, int orderC, int mode,
                      void *workspace, size_t workspace_bytes, void *stream) {
  PackedLayout L;
  if (m < 0 || m > MIPGEMM_MAX_DIM) return -1;
  if (!packed_layout(k, n, &L)) return n < 0 || n > MIPGEMM_MAX_DIM ? -2 : -3;
  if (!packed || reinterpret_cast<uintptr_t>(packed) % 16 != 0) return -7;
  const uint8_t *body = static_cast<const uint8_t *>(packed);
  const int rc = mip::run_gemm(a_unsigned, 0, 0, 1.0f, m, n, k, A, lda, orderA, body, L.kp,
                               MIPGEMM_COL_MAJOR, C, ldc, orderC, mode, workspace, workspace_bytes,
                               stream, mip::Batch(),
                               reinterpret_cast<const int32_t *>(body + L.sums_at));
  if (rc >= -7) return rc;    // success, a hipError_t, or one of the first seven arguments
  return rc + 2;              // C, ldc, orderC, mode, workspace: two places earlier here
}

int mipgemm_s8s8s32_packed(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                           const void *packed, int32_t *C, int64_t ldc, int orderC, int mode,
                           void *workspace, size_t workspace_bytes, void *stream) {
  return run_packed(0, m, n, k, A, lda, orderA, packed, C, ldc, orderC, mode, workspace,
                    workspace_bytes, stream);
}

int mipgemm_u8s8s32_packed(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                           const void *packed, int32_t *C, int64_t ldc, int orderC, int mode,
                           void *workspace, size_t workspace_bytes, void *stream) {
  return run_packed(1, m, n, k, A, lda, orderA, packed, C, ldc, orderC, mode, workspace,
                    workspace_bytes, stream);
}

int mipgemm_s8u8s32(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc, int orderC,
                    int mode, void *workspace, size_t workspace_bytes, void *stream) {
  return mip::run_gemm(0, 1, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
             workspace_bytes, stream);
}

// Strided batch of equal-shape problems in one launch (one grid z-slice per problem).
static int run_batched(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k, const void *A,
                       int64_t lda, int orderA, int64_t strideA, const void *B, int64_t ldb,
                       int orderB, int64_t strideB, int32_t *C, int64_t ldc, int orderC,
                       int64_t strideC, int64_t batch, int mode, void *workspace,
                       size_t workspace_bytes, void *stream) {
  // the shared validation numbers its arguments as the single-problem entry points do:
  // map them onto this prototype (strides and batch shift everything after orderA)
  static const int renumber[17] = {0, 1, 2, 3, 4, 5, 6, 8, 9, 10, 12, 13, 14, 17, 18, 19, 20};
  Problem probe;
  const int base = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
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
  return mip::run_gemm(a_unsigned, b_unsigned, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
             workspace, workspace_bytes, stream, b);
}

int mipgemm_s8s8s32_batched(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda,
                            int orderA, int64_t strideA, const int8_t *B, int64_t ldb, int orderB,
                            int64_t strideB, int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode, void *workspace, size_t workspace_bytes,
                            void *stream) {
  return run_batched(0, 0, m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB, C, ldc, orderC,
                     strideC, batch, mode, workspace, workspace_bytes, stream);
}

int mipgemm_u8s8s32_batched(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda,
                            int orderA, int64_t strideA, const int8_t *B, int64_t ldb, int orderB,
                            int64_t strideB, int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode, void *workspace, size_t workspace_bytes,
                            void *stream) {
  return run_batched(1, 0, m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB, C, ldc, orderC,
                     strideC, batch, mode, workspace, workspace_bytes, stream);
}

int mipgemm_s8u8s32_batched(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda,
                            int orderA, int64_t strideA, const uint8_t *B, int64_t ldb, int orderB,
                            int64_t strideB, int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode, void *workspace, size_t workspace_bytes,
                            void *stream) {
  return run_batched(0, 1, m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB, C, ldc, orderC,
                     strideC, batch, mode, workspace, workspace_bytes, stream);
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
  return mip::run_gemm(a_unsigned, b_unsigned, 1, scale, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
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

static size_t recommended_workspace(int64_t m, int64_t n, int64_t k, int orderA, int orderB,
                                    int orderC, int out_float) {
  // Operands that are 16-byte aligned with k a multiple of 64 go straight from their own
  // storage through LDS into the matrix cores; the others are packed first when that pays.
  // Either way, a problem with too few tiles for the chip splits k, and the ranges meet in
  // slots of partial sums when there is room for them.
  if (m < 0 || n < 0 || k < 0 || m > MIPGEMM_MAX_DIM || n > MIPGEMM_MAX_DIM || k > MIPGEMM_MAX_DIM)
    return 0;
  if (!mip::order_ok(orderA) || !mip::order_ok(orderB) || !mip::order_ok(orderC)) return 0;
  if (m == 0 || n == 0 || k == 0) return 0;
  // the tightest leading dimensions of these orders, on 16-byte aligned pointers
  Problem p;
  const void *fake = reinterpret_cast<const void *>(uintptr_t(4096));
  if (validate_and_normalise(0, 0, m, n, k, fake, orderA == MIPGEMM_ROW_MAJOR ? k : m, orderA, fake,
                             orderB == MIPGEMM_ROW_MAJOR ? n : k, orderB,
                             reinterpret_cast<int32_t *>(uintptr_t(4096)),
                             orderC == MIPGEMM_ROW_MAJOR ? n : m, orderC, MIPGEMM_OVERWRITE, nullptr, 0,
                             &p) != 0)
    return 0;
  p.ws = const_cast<void *>(fake);  // "there is a workspace": the plan may count on slots
  p.ws_bytes = ~size_t(0) / 2;
  p.out_float = out_float;
  size_t total = 0;
  mip::Plan plan = mip::choose_plan(p);
  if (mip::packing_size_ok(p.m, p.n, p.k) && mip::packing_pays(p, plan)) {
    total = (mip::packed_bytes(p.m, p.n, p.k) + 255) / 256 * 256;
    const int64_t kp = mip::padded_k(p.k);
    p.a_sm = p.b_sn = kp;
    p.a_sk = p.b_sk = 1;
    p.k = kp;
    p.rows_padded_to_256 = true;
    plan = mip::choose_plan(p);
  }
  return total + mip::splitk_slot_bytes(p, plan);
}

// Requantised int8 output (the paper's quantization scheme, Section 7.3, applied to the
// product).  Same arguments and numbering as the f32 entry points; overwrite only.
static int run_q8(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k, const void *A,
                  int64_t lda, int orderA, const void *B, int64_t ldb, int orderB, int8_t *C,
                  int64_t ldc, int orderC, int mode, void *workspace, size_t workspace_bytes,
                  void *stream, float scale) {
  Problem p;
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB, C,
                                  ldc, orderC, mode, workspace, workspace_bytes, &p);
  if (rc != 0) return rc;
  if (mode != MIPGEMM_OVERWRITE) return -13;  // a quantized output has no running sum
  if (!(scale == scale) || scale - scale != 0.0f) return -17;
  return mip::run_gemm(a_unsigned, b_unsigned, 2, scale, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
                       orderC, mode, workspace, workspace_bytes, stream);
}

int mipgemm_s8s8s8(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                   const int8_t *B, int64_t ldb, int orderB, int8_t *C, int64_t ldc, int orderC,
                   int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_q8(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                workspace_bytes, stream, scale);
}

int mipgemm_u8s8s8(int64_t m, int64_t n, int64_t k, const uint8_t *A, int64_t lda, int orderA,
                   const int8_t *B, int64_t ldb, int orderB, int8_t *C, int64_t ldc, int orderC,
                   int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_q8(1, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                workspace_bytes, stream, scale);
}

int mipgemm_s8u8s8(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                   const uint8_t *B, int64_t ldb, int orderB, int8_t *C, int64_t ldc, int orderC,
                   int mode, void *workspace, size_t workspace_bytes, void *stream, float scale) {
  return run_q8(0, 1, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode, workspace,
                workspace_bytes, stream, scale);
}

size_t mipgemm_workspace_size(int64_t m, int64_t n, int64_t k, int orderA, int orderB, int orderC) {
  return recommended_workspace(m, n, k, orderA, orderB, orderC, 0);
}

size_t mipgemm_workspace_size_f32(int64_t m, int64_t n, int64_t k, int orderA, int orderB, int orderC) {
  return recommended_workspace(m, n, k, orderA, orderB, orderC, 1);
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
  if (code == MIPGEMM_ERR_STATIC_SCRATCH)
    return "the problem needs more scratch memory than the library's static buffer holds";
  if (code > 0) return hipGetErrorString(static_cast<hipError_t>(code));
  return "unknown mipgemm error code";
}

const char *mipgemm_variant_name_for_mode(int64_t m, int64_t n, int64_t k, int64_t lda, int orderA,
                                          int64_t ldb, int orderB, int64_t ldc, int orderC,
                                          int a_unsigned, int b_unsigned, int aligned16, int mode) {
  Problem p;
  // stand-in addresses that only carry the alignment
  const void *fake = reinterpret_cast<const void *>(aligned16 ? uintptr_t(4096) : uintptr_t(4097));
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, fake, lda, orderA, fake, ldb,
                                  orderB, reinterpret_cast<int32_t *>(uintptr_t(4096)), ldc,
                                  orderC, mode, nullptr, 0, &p);
  if (rc != 0) return "invalid";
  return mip::plan_name(mip::choose_plan(p));
}

const char *mipgemm_variant_name(int64_t m, int64_t n, int64_t k, int64_t lda, int orderA,
                                 int64_t ldb, int orderB, int64_t ldc, int orderC, int a_unsigned,
                                 int b_unsigned, int aligned16) {
  return mipgemm_variant_name_for_mode(m, n, k, lda, orderA, ldb, orderB, ldc, orderC, a_unsigned,
                                       b_unsigned, aligned16, MIPGEMM_OVERWRITE);
}

const char *mipgemm_variant_name_with_workspace(int64_t m, int64_t n, int64_t k, int64_t lda,
                                                int orderA, int64_t ldb, int orderB, int64_t ldc,
                                                int orderC, int a_unsigned, int b_unsigned,
                                                int aligned16) {
  Problem p;
  const void *fake = reinterpret_cast<const void *>(aligned16 ? uintptr_t(4096) : uintptr_t(4097));
  int rc = validate_and_normalise(a_unsigned, b_unsigned, m, n, k, fake, lda, orderA, fake, ldb,
                                  orderB, reinterpret_cast<int32_t *>(uintptr_t(4096)), ldc,
                                  orderC, MIPGEMM_OVERWRITE, nullptr, 0, &p);
  if (rc != 0) return "invalid";
  const mip::Plan plan = mip::choose_plan(p);
  if (!mip::packing_pays(p, plan)) return mip::plan_name(plan);
  // the plan for the packed operands: aligned, k-contiguous, k padded
  const int64_t kp = mip::padded_k(p.k);
  p.A = p.B = reinterpret_cast<const void *>(uintptr_t(4096));
  p.a_sm = p.b_sn = kp;
  p.a_sk = p.b_sk = 1;
  p.k = kp;
  p.rows_padded_to_256 = true;
#define MIP_NAME(x) {x, "packed+" x}
  static const char *const names[][2] = {
      MIP_NAME("mfma_dma256"), MIP_NAME("mfma_dma128"), MIP_NAME("mfma_dma64"),
      MIP_NAME("mfma_dma64x256"), MIP_NAME("mfma_dma256x64"), MIP_NAME("mfma_dma64x128"),
      MIP_NAME("mfma_dma128x64"), MIP_NAME("mfma_dma256_k128"), MIP_NAME("mfma_dma128_k128"),
      MIP_NAME("mfma_dma128_k128_split"), MIP_NAME("mfma_dma256_k128_ragged"), MIP_NAME("mfma_slab16"),
      MIP_NAME("mfma_slab32"), MIP_NAME("mfma_slab64")};
#undef MIP_NAME
  const char *base = mip::plan_name(mip::choose_plan(p));
  for (const auto &nm : names)
    if (!std::strcmp(nm[0], base)) return nm[1];
  return "packed";
}

}  // extern "C"
