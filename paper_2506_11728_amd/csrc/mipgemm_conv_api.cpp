// C-ABI entry points of the steps around the GEMM: the convolution lowering (paper Section
// 7.2) and the pre-packing of a weight matrix (Section 4.1).  Host only.
#include <cstdlib>
#include <cstring>

#include "api_internal.h"
#include "tuning.h"

using mip::Problem;
using mip::order_ok;

// ---------------------------------------------------------------------------
// convolution by lowering (paper Section 7.2)
// ---------------------------------------------------------------------------
namespace {

struct ConvCall {
  mip::ConvGeom geom;
  int64_t rows;  // b * h_o * w_o: the GEMM's n
  int64_t k;     // h_f * w_f * c_i
  int64_t kp;    // row pitch of a written-out augmented matrix: k padded (with zeros) to whole k blocks
};

int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

// The written-out route's workspace: the augmented matrix, rows in whole tiles of 256 (only
// the real ones are written) with pitch kp, then the filters re-pitched to kp the same way.
size_t written_out_bytes(const ConvCall &c, int64_t co) {
  return static_cast<size_t>((round_up(c.rows, 256) + round_up(co, 256)) * c.kp);
}

// 0 and `out`, or the negative number of the first bad size argument; has_co is false for
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
  out->kp = out->k >= 1024 ? round_up(out->k, 128) : round_up(out->k, 64);
  return 0;
}

// the GEMM the convolution is lowered to, in the kernels' terms: the row-major C is O
// seen as (b h_o w_o) x c_o, its A the augmented matrix, its B the filters (k contiguous)
Problem conv_problem(const ConvCall &c, int64_t co, const void *F, const void *I, void *O, int mode,
                     bool implicit, const void *M, int out_float = 0, float scale = 1.0f) {
  Problem p;
  p.m = c.rows; p.n = co; p.k = c.k;
  // written out: M holds the matrix and, behind its round_up(rows, 256) rows, the filters,
  // both with pitch kp and zeros from k on
  p.A = implicit ? I : M; p.a_sm = implicit ? c.k : c.kp; p.a_sk = 1; p.a_unsigned = 1;
  p.B = implicit ? F : static_cast<const uint8_t *>(M) + round_up(c.rows, 256) * c.kp;
  p.b_sk = 1; p.b_sn = implicit ? c.k : c.kp; p.b_unsigned = 0;
  if (!implicit) {
    p.k = c.kp;
    p.rows_padded_to_256 = true;
  }
  p.C = static_cast<int32_t *>(O); p.ldc = co;
  p.accumulate = mode == MIPGEMM_ACCUMULATE;
  p.out_float = out_float; p.scale = scale;
  p.conv = nullptr;
  return p;
}

// How a convolution is carried out.
enum Route {
  ROUTE_TILES,   // a direct-to-LDS tile kernel gathers the augmented matrix (channels in 16-byte runs)
  ROUTE_ROWS,    // the row-segment kernel gathers it (any channel count, small k)
  ROUTE_IM2COL   // the augmented matrix is written to the workspace, then a plain GEMM
};

// The tuning value MIPGEMM_CONV pins a route for tests and tuning: "im2col" the written-out one, "rows" the
// row-segment kernel where it can serve.
Route conv_route(const ConvCall &c, Problem p, mip::Plan *plan) {
  const int pinned = mip::tuning().conv;
  if (pinned == 1) return ROUTE_IM2COL;
  if (p.m == 0 || p.n == 0) return ROUTE_IM2COL;
  p.conv = &c.geom;
  if (pinned == 2 && mip::conv_rows_eligible(p)) return ROUTE_ROWS;
  *plan = mip::choose_plan(p);
  if (plan->kind == mip::KIND_DMA) return ROUTE_TILES;
  // The row-segment kernel stages the image once per block of 64 filters: with many filters
  // the written-out route wins (measured at batch 32: 576 filters 1 x 1 on 28 x 28 x 96,
  // 50 against 20 us; 240 on 14 x 14 x 40, 18 against 15; 144 on 56 x 56 x 24, 28 against 30).
  const int64_t filter_blocks = (p.n + 63) / 64;
  const bool rows_pays = filter_blocks <= 2 || (filter_blocks == 3 && c.geom.wo >= 48);
  return rows_pays && mip::conv_rows_eligible(p) ? ROUTE_ROWS : ROUTE_IM2COL;
}

}  // namespace

extern "C" {

static size_t conv_workspace_for(const void *fake, int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                 int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad) {
  ConvCall c;
  if (conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c) != 0) return 0;
  if (c.rows == 0 || co == 0) return 0;
  mip::Plan plan;
  if (conv_route(c, conv_problem(c, co, fake, fake, const_cast<void *>(fake), MIPGEMM_OVERWRITE,
                                 true, nullptr), &plan) != ROUTE_IM2COL)
    return 0;
  return written_out_bytes(c, co);
}

size_t mipgemm_conv_workspace_size(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                   int64_t hf, int64_t wf, int64_t stride, int64_t pad) {
  return conv_workspace_for(reinterpret_cast<const void *>(uintptr_t(4096)), b, hi, wi, ci, co, hf,
                            wf, stride, pad);
}

size_t mipgemm_conv_workspace_size_unaligned(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                             int64_t co, int64_t hf, int64_t wf, int64_t stride,
                                             int64_t pad) {
  return conv_workspace_for(reinterpret_cast<const void *>(uintptr_t(4097)), b, hi, wi, ci, co, hf,
                            wf, stride, pad);
}

const char *mipgemm_conv_variant_name(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                      int64_t hf, int64_t wf, int64_t stride, int64_t pad) {
  ConvCall c;
  if (conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c) != 0) return "invalid";
  if (c.rows == 0 || co == 0) return "none";
  const void *fake = reinterpret_cast<const void *>(uintptr_t(4096));
  mip::Plan plan;
  const Route route = conv_route(
      c, conv_problem(c, co, fake, fake, const_cast<void *>(fake), MIPGEMM_OVERWRITE, true, nullptr),
      &plan);
  if (route == ROUTE_ROWS) return "implicit:rows";
  const bool implicit = route == ROUTE_TILES;
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
                    void *stream, const int32_t *filter_sums = nullptr) {
  ConvCall c;
  int rc = conv_sizes(b, hi, wi, ci, co, true, hf, wf, stride, pad, &c);
  if (rc != 0) return rc;
  if (!F && co > 0) return -10;
  if (!I && b > 0) return -11;
  if (!O && c.rows > 0 && co > 0) return -12;
  if (mode != MIPGEMM_OVERWRITE && mode != MIPGEMM_ACCUMULATE) return -13;
  if (out_float == 2 && mode != MIPGEMM_OVERWRITE) return -13;  // a quantized output has no running sum
  if (out_float && (!(scale == scale) || scale - scale != 0.0f)) return -17;  // NaN or infinity
  if (c.rows == 0 || co == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  mip::Plan plan;
  Problem p = conv_problem(c, co, F, I, O, mode, true, nullptr, out_float, scale);
  const Route route = conv_route(c, p, &plan);
  p.conv = &c.geom;
  p.ksum = filter_sums;  // the filters are the signed B of the lowered product: one sum per column
  if (route == ROUTE_TILES) return static_cast<int>(mip::launch_dma(p, plan.shape, plan.splits, s));
  if (route == ROUTE_ROWS) return static_cast<int>(mip::launch_conv_rows(p, s));
  const size_t need = written_out_bytes(c, co);
  if (!workspace) return -14;
  if (workspace_bytes < need) return -15;
  // the matrix and the filters, both with pitch kp and the k tail zeroed, so that the
  // direct-to-LDS kernels can stream them whatever k and the alignment of F are
  uint8_t *Mp = static_cast<uint8_t *>(workspace);
  uint8_t *Fp = Mp + round_up(c.rows, 256) * c.kp;
  hipError_t e = mip::launch_im2col(c.geom, c.rows, c.k, I, Mp, c.kp, s, c.kp);
  if (e != hipSuccess) return static_cast<int>(e);
  p = conv_problem(c, co, F, I, O, mode, false, Mp, out_float, scale);
  p.ksum = filter_sums;
  if (c.kp == c.k && reinterpret_cast<uintptr_t>(F) % 16 == 0) {
    p.B = F;  // the filters can be streamed where they are
    p.b_sn = c.k;
    p.rows_padded_to_256 = false;
  } else {
    e = mip::launch_pack_b(c.k, co, reinterpret_cast<const uint8_t *>(F), c.k, true, Fp, c.kp, s, c.kp);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  return static_cast<int>(mip::launch_plan(p, mip::choose_plan(p), s));
}

int mipgemm_conv_s8u8s32(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co, int64_t hf,
                         int64_t wf, int64_t stride, int64_t pad, const int8_t *F, const uint8_t *I,
                         int32_t *O, int mode, void *workspace, size_t workspace_bytes,
                         void *stream) {
  return run_conv(0, 1.0f, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream);
}

int mipgemm_conv_filter_sums(int64_t co, int64_t k, const int8_t *F, int32_t *sums, void *stream) {
  if (co < 0 || co >= ((int64_t)1 << 31)) return -1;
  if (k < 0 || k >= ((int64_t)1 << 31)) return -2;
  if (!F && co > 0 && k > 0) return -3;
  if (!sums && co > 0) return -4;
  return static_cast<int>(mip::launch_column_sums(k, co, reinterpret_cast<const uint8_t *>(F), k, sums,
                                                  static_cast<hipStream_t>(stream)));
}

int mipgemm_conv_s8u8s32_with_sums(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                   int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                                   const int8_t *F, const uint8_t *I, int32_t *O, int mode,
                                   void *workspace, size_t workspace_bytes, void *stream,
                                   const int32_t *filter_sums) {
  if (!filter_sums && co > 0) return -17;
  return run_conv(0, 1.0f, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream, filter_sums);
}

int mipgemm_conv_s8u8f32_with_sums(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co,
                                   int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                                   const int8_t *F, const uint8_t *I, float *O, int mode,
                                   void *workspace, size_t workspace_bytes, void *stream, float scale,
                                   const int32_t *filter_sums) {
  if (!filter_sums && co > 0) return -18;
  return run_conv(1, scale, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream, filter_sums);
}

int mipgemm_conv_s8u8s8(int64_t b, int64_t hi, int64_t wi, int64_t ci, int64_t co, int64_t hf,
                        int64_t wf, int64_t stride, int64_t pad, const int8_t *F, const uint8_t *I,
                        int8_t *O, int mode, void *workspace, size_t workspace_bytes, void *stream,
                        float scale, const int32_t *filter_sums) {
  return run_conv(2, scale, b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, workspace,
                  workspace_bytes, stream, filter_sums);
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

}  // extern "C"
