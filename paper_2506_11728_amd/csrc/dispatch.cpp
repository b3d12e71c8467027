// Which kernel serves which problem: eligibility, tile shape, k ranges.  Host only.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "mip_internal.h"
#include "tuning.h"

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
    case KIND_DMA_K128: return plan.shape == SHAPE_128 ? "mfma_dma128_k128" : "mfma_dma256_k128";
    case KIND_DMA_K128_SPLIT: return plan.shape == SHAPE_256 ? "mfma_dma256_k128_ragged" : "mfma_dma128_k128_split";
    case KIND_SLAB: return plan.splits == 4 ? "mfma_slab64" : (plan.splits == 2 ? "mfma_slab32" : "mfma_slab16");
    default: return "?";
  }
}

// The tuning value MIPGEMM_VARIANT pins the kernel (tuning and tests): "simple", "dma256k128",
// "dma128k128" (the same kernel on 128 x 128 tiles), "dma128k128split" (its general form with k ranges), "dma256k128ragged" (the general form on 256 x 256 tiles),
// "slab16" / "slab32" (the skinny-m kernel with that slab width),
// "tile<shape>" (register-staged) or "dma<shape>" (direct-to-LDS) with <shape> one of
// 256, 128, 64, 64x256, 256x64, 64x128, 128x64.  A dma variant only applies to problems it is
// eligible for; others fall back to the staged kernel of the same shape.
// MIPGEMM_SPLITK pins the number of k ranges of the tile kernels.
static int forced_splits() { return tuning().splitk; }

// k ranges for the 128 x 128 tiles with 128-deep blocks: workgroups for about three quarters
// of the compute units, at most eight ranges (every range adds a whole C through atomics), each
// of at least eight blocks.  Measured best, ranges at tiles: 6-8 at 16, 6 at 24, 4 at 36 to 52,
// 3-4 at 64, 2 at 96.
static int k128_ranges(const Problem &p) {
  if (forced_splits() > 0) return forced_splits();
  const int64_t tiles = ((p.m + 127) / 128) * ((p.n + 127) / 128);
  const int64_t blocks = p.k / 128;
  int64_t sp = (3 * compute_units() / 4 + tiles / 2) / tiles;
  if (sp > 8) sp = 8;
  if (sp > blocks / 8) sp = blocks / 8;
  return sp > 1 ? (int)sp : 1;
}

static bool forced_plan(const Problem &p, Plan *plan) {
  const char *e = tuning().variant;
  if (!*e) return false;
  if (!std::strcmp(e, "simple")) { *plan = {KIND_SIMPLE, SHAPE_64, 1}; return true; }
  if (!std::strcmp(e, "dma256k128")) {
    if (!dma_k128_eligible(p)) return false;
    *plan = {KIND_DMA_K128, SHAPE_256, 1};
    return true;
  }
  if (!std::strcmp(e, "dma128k128")) {
    if (!dma_k128_eligible(p, true)) return false;
    *plan = {KIND_DMA_K128, SHAPE_128, 1};
    return true;
  }
  if (!std::strcmp(e, "dma128k128split")) {
    if (!dma_k128_split_eligible(p)) return false;
    *plan = {KIND_DMA_K128_SPLIT, SHAPE_128, k128_ranges(p)};
    return true;
  }
  if (!std::strcmp(e, "dma256k128ragged")) {
    if (!dma_k128_split_eligible(p, true)) return false;
    *plan = {KIND_DMA_K128_SPLIT, SHAPE_256, 1};
    return true;
  }
  if (!std::strcmp(e, "slab16") || !std::strcmp(e, "slab32") || !std::strcmp(e, "slab64")) {
    const int nt = e[4] == '6' ? 4 : (e[4] == '3' ? 2 : 1);
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

hipError_t allow_dynamic_lds(const void *kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  struct Granted { const void *kernel; int device; size_t bytes; };
  static std::mutex lock;
  static std::vector<Granted> granted;  // a few dozen kernels at most
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> guard(lock);
  for (Granted &g : granted)
    if (g.kernel == kernel && g.device == device) {
      if (g.bytes >= bytes) return hipSuccess;
      e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
      if (e == hipSuccess) g.bytes = bytes;
      return e;
    }
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) granted.push_back({kernel, device, bytes});
  return e;
}

// Compute units of the current device, asked once; 256 (an MI355X) where no device answers,
// as on a build host that only names kernels.
int64_t compute_units() {
  static std::once_flag once;
  static int64_t count = 256;
  std::call_once(once, [] {
    int device = 0, n = 0;
    if (hipGetDevice(&device) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && n > 0)
      count = n;
    (void)hipGetLastError();  // a missing device must not surface in a later call
  });
  return count;
}

// over all problems of a batch: what the chip sees is their sum
static int64_t tile_count(const Problem &p, Shape s) {
  return ((p.m + kShapeRows[s] - 1) / kShapeRows[s]) * ((p.n + kShapeCols[s] - 1) / kShapeCols[s]) *
         (p.batch > 1 ? p.batch : 1);
}

size_t splitk_slot_bytes(const Problem &p, const Plan &plan) {
  if (plan.kind != KIND_DMA || plan.splits < 2 || !p.out_float) return 0;  // (int32 outputs add into C)
  const int64_t bm = kShapeRows[plan.shape], bn = kShapeCols[plan.shape];
  const int64_t tiles = ((p.m + bm - 1) / bm) * ((p.n + bn - 1) / bn) * (p.batch > 1 ? p.batch : 1);
  const double bytes = (double)tiles * (double)plan.splits * (double)(bm * bn * 4);
  return bytes < 1.0e15 ? (size_t)bytes : 0;
}

Plan choose_plan(const Problem &p) {
  const int64_t kComputeUnits = compute_units();
  if (p.m == 0 || p.n == 0) return {KIND_NONE, SHAPE_64, 1};
  // (the zero fill writes words; an int8 output of an empty sum goes through the simple kernel)
  if (p.k == 0) return {p.accumulate ? KIND_NONE : (p.out_float == 2 ? KIND_SIMPLE : KIND_FILL), SHAPE_64, 1};
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
    const Shape rect = (!p.conv && p.b_sn == 1 && p.a_sk == 1)   ? SHAPE_64X128
                       : (!p.conv && p.a_sm == 1 && p.b_sk == 1) ? SHAPE_128X64
                                                                 : (p.m >= p.n ? SHAPE_128X64 : SHAPE_64X128);
    const int64_t ranges = p.k / 512 > 1 ? p.k / 512 : 1;
    auto enough = [&](Shape wide, int64_t short_side) {
      const int64_t t = tile_count(p, wide);
      return t >= kComputeUnits || (short_side <= 16 && !p.out_float && t * ranges >= kComputeUnits);
    };
    // (With k under 512 a workgroup holds one to eight k blocks; 64 x 64 tiles then need
    // little LDS, many fit a compute unit, and they overtake the wide tiles:
    // (64, 100352, 64) 10.9 -> 9.4 us, (64, 100352, 256) 12.4 -> 11.7 us.)
    // (From 32 rows on, a weight matrix that does not fit the L2 caches streams better through
    // 64 x 128 tiles, whole 128-byte lines of a row-major B, than through 64 x 64 ones; measured
    // cold, us: (32, 11008, 4096) 18.9 -> 16.5, (64, 11008, 4096) 20.7 -> 18.7, (32, 4096, 11008)
    // 18.9 -> 15.3, (64, 4096, 11008) 21.5 -> 18.9; warm within 0.5 us either way; at
    // (64, 4096, 4096) the 64 x 64 tiles stay ahead, 11.6 against 12.7.  A k-contiguous B has no
    // lines to complete: (64, 11008, 4096) 13.3/19.2 us warm/cold on 64 x 64, 16.2/20.8 on 64 x 128.)
    if (p.m <= 64 && p.n > 128)
      sh = p.k >= 512 && enough(SHAPE_64X256, p.m)
               ? SHAPE_64X256
               : (p.m >= 32 && p.k >= 512 && p.b_sn == 1 && p.n * p.k >= ((int64_t)32 << 20) &&
                          dma_eligible(p, SHAPE_64X128)
                      ? SHAPE_64X128
                      : SHAPE_64);
    else if (p.n <= 64 && p.m > 128) sh = p.k >= 512 && enough(SHAPE_256X64, p.n) ? SHAPE_256X64 : SHAPE_64;
    // A large tile buys operand reuse, which only a long k turns into time: with a short
    // k the problem is a stream that ends in the write of C, and small tiles, several
    // workgroups to a compute unit, overlap that write with the next tile's loads.
    // Between 128 x 128 (too few tiles) and 64 x 64 (64 operations per operand byte,
    // which the L2 caches cannot feed) sit the 8192-element tiles, long side along the
    // longer dimension of C.
    // (One 256 x 256 workgroup fills a compute unit: a few tiles more than there are
    // compute units cost a second round almost in full, which 128 x 128 tiles, two
    // workgroups to a compute unit, do not.  Measured at k = 4096: 289 tiles 121 us
    // against 110, 324 tiles 124 against 125, 400 tiles 132 against 150.)
    else if (p.k >= 1024 && tile_count(p, SHAPE_256) >= 192 &&
             !(tile_count(p, SHAPE_256) > kComputeUnits && tile_count(p, SHAPE_256) <= 320))
      sh = SHAPE_256;
    // (128 x 128 tiles from three quarters of a round on: measured cold against the
    // 8192-element tiles, us: (128, 25088, 1152) 15.2 -> 12.6, (256, 12544, 1152) 14.8 -> 11.2,
    // (768, 4096, 2048) 17.9 -> 13.1, (1024, 3072, 3072) 26.6 -> 23.4, (1024, 3072, 768) 8.2 -> 7.9.)
    else if (p.k >= 512 && !p.conv && tile_count(p, SHAPE_128) >= 192) sh = SHAPE_128;
    // (The long side of an 8192-element tile goes along a row-major B, whose rows it then
    // fetches in whole 128-byte lines, or down a column-major A; with both operands
    // k-contiguous or both strided, along the longer dimension of C.  (3072, 1024, 768)
    // row-major: 128 x 64 8.9 us cold, 64 x 128 8.0; (6272, 256, 2304) 15.4 and 13.0.  They
    // serve from three quarters of a round of tiles on: (256, 6272, 2304) 19.9 us on 64 x 64
    // tiles, 13.3 on 196 tiles of 64 x 128.)
    // (A gathered convolution keeps the order it was measured with: 8192-element tiles from a
    // whole round on, long side along the longer dimension, then 128 x 128 tiles.)
    else if (p.k >= 512 && tile_count(p, rect) >= (p.conv ? kComputeUnits : 192) && dma_eligible(p, rect))
      sh = rect;  // (measured on the direct-to-LDS kernels only)
    else if (p.k >= 512 && tile_count(p, SHAPE_128) >= 192) sh = SHAPE_128;
    else sh = SHAPE_64;
    // deep k blocks pay off once the k loop is long enough to amortise their prologue
    // A few rows of A against a k-contiguous B is one pass over B with nothing to
    // share: a workgroup per 16-column slab does it in one launch, without atomics.
    // (A row-major B would reach each slab in 16-byte pieces of its cache lines,
    // which the tiled kernels, with their 64-byte pieces and split k, do better.)
    // The same kernel serves short k, where the tiled kernels cannot split k
    // and 64-column tiles leave most compute units idle.
    // (Adding into an int32 C that already holds values needs no zero-fill launch: with a k
    // long enough to split, the tiles then win or tie.  Measured, us warm/cold, slab against
    // tiles: (16, 4096, 4096) 6.4/9.5 against 4.7/7.0, (1, 1024, 2048) 3.7/4.7 against
    // 3.3/4.0, (64, 4096, 1024) 5.4/6.5 against 4.5/5.2, (16, 16384, 4096) 16.1/21.9 against
    // 15.0/18.2, (1, 11008, 4096) 10.4/12.5 against 10.5/12.2.  At k = 1024 only from 16
    // rows on: (1, 4096, 1024) 2.9/3.5 against 3.4/4.1, (16, 8192, 1024) 4.2/5.7 against 3.9/4.7;
    // with fewer rows from k = 1536: (8, 4096, 1536) 4.0/5.1 against 3.5/4.3,
    // (4, 16384, 1536) 6.2/8.4 against 4.6/8.2.)
    const bool adds_in_place = p.accumulate && !p.out_float && p.k >= (p.m >= 16 ? 1024 : 1536);
    const bool slab_ok = p.m <= 64 && !adds_in_place && slab_eligible(p, 1);
    // Slabs of 32 columns re-read A half as often and need half the workgroups; they win
    // (warm and cold) wherever they fill the compute units' rounds as evenly as slabs of 16 do:
    // n = 8192 (256 slabs of 32: one round) and 16384, not 11008 (344: two rounds, the second
    // a third full) nor 4096 (128: half a round).  Measured, us warm/cold, m = 1, k = 4096:
    // n = 16384 15.7/19.7 -> 12.5/18.0; m = 16: 18.5/21.9 -> 14.7/19.6.
    auto round_fill = [&](int64_t slabs) {
      return (double)slabs / (double)((slabs + kComputeUnits - 1) / kComputeUnits * kComputeUnits);
    };
    const bool wide_slabs = slab_eligible(p, 2) && round_fill(p.n / 32) >= round_fill(p.n / 16) - 0.02;
    // "short k": the slab kernel still wins where the tiles, too few to fill the chip, would
    // have to split k (a zero-fill launch plus atomics): up to k = 4096 at m <= 16, 2048 at 32,
    // 1024 at 64; with a row-major B (16-byte pieces of every line per slab) only up to 2048,
    // cold it loses beyond ((1, 4096, 3072): 11.6 against 8.5 us).  Measured, us warm/cold:
    // (1, 1024, 2048) 4.9/5.6 -> 3.6/4.5, (16, 2048, 2048) 5.3/6.1 -> 4.5/5.5,
    // (64, 4096, 1024) 6.3/7.2 -> 5.1/5.7.
    const bool short_k = p.k * (p.m > 16 ? p.m : 16) <= 65536 && (p.b_sk == 1 || p.k <= 2048);
    // Slabs of 64 columns re-read A a quarter as often, which is what several rows of A cost a
    // narrow slab; they need n / 64 workgroups to be enough.  Measured on a k-contiguous B, us
    // warm/cold against the narrower choice: (16, 11008, 4096) 14.2/16.2 -> 12.1/15.1,
    // (16, 16384, 4096) 14.8/19.6 -> 13.2/18.0, (16, 32000, 4096) 26.7/33.0 -> 22.6/31.8,
    // (1, 16384, 4096) 12.6/18.3 -> 12.3/17.1; not (1, 11008, 4096) 10.4/12.2 -> 10.5/12.8, nor
    // n = 4096 at any m (64 workgroups: (16, 4096, 4096) 6.3/8.2 -> 11.2/13.1).
    const bool slabs_of_64 = slab_eligible(p, 4) && p.n / 64 >= 160 && (p.m > 4 || p.n / 64 >= 256);
    if (slab_ok && p.b_sk == 1 && p.m <= 16 && p.n / 16 >= 192)
      plan = {KIND_SLAB, SHAPE_64, slabs_of_64 ? 4 : (wide_slabs ? 2 : 1)};
    // (Float output cannot split k at all, sums of floats not being combined out of order:
    // there the slab kernel takes every such problem, whatever k.  Measured, us warm/cold:
    // (16, 2048, 8192) 17.8/29.2 -> 9.7/11.2, with a row-major B 17.7/35.3 -> 10.5/26.6;
    // (1, 4096, 4096) row-major B 10.5/18.5 -> 7.2/14.5.)
    // (With a workspace a float output splits k through slots of partial sums, and then the
    // tiles win here as they do for an int32 output: (64, 4096, 4096) 15.7 -> 9.4 us,
    // (16, 4096, 4096) 10.8 -> 9.2 us.)
    else if (slab_ok && (short_k || (p.out_float && !p.ws)) && tile_count(p, SHAPE_64) < kComputeUnits / 2 &&
             p.n / 16 >= 64)
      plan = {KIND_SLAB, SHAPE_64, 1};
    // A very long k over few tiles: the 128 x 128 tiles with 128-deep blocks, k in ranges.
    // The 64 x 64 tiles chosen above for such a shape (enough of them to need no split) run
    // at 64 operations per operand byte; the wider tile halves the bytes, and the ranges give
    // the compute units their workgroups.  Measured warm/cold, us, against the choice above:
    // (768, 768, 8192) 22.8/31.0 -> 18.8/22.6, (512, 1568, 8192) 25.4/34.6 -> 21.5/25.2,
    // (1024, 1024, 16384) 46.5/60.0 -> 32.7/37.4, (768, 2048, 16384) 54.6/73.4 -> 45.3/51.4,
    // (512, 512, 16384) 19.0/23.1 -> 17.7/20.7; accumulating (no zero-fill launch) already from
    // k = 6144: (768, 768, 6144) 18.1/18.5 -> 14.7/17.0, (512, 1568, 6144) 20.1/26.8 -> 16.9/19.8.
    // Not below: at k = 4608 the atomics cost what the ranges save, (1024, 1024, 4608)
    // 13.2/15.4 against 19.8/22.0, (512, 1568, 4608) 14.7/16.7 against 16.7/20.0.
    else if (!p.out_float && p.m > 64 && p.n > 64 && p.k >= (p.accumulate ? 6144 : 8192) &&
             tile_count(p, SHAPE_128) >= 16 &&
             tile_count(p, SHAPE_128) <= 3 * kComputeUnits / 8 && dma_k128_split_eligible(p))
      plan = {KIND_DMA_K128_SPLIT, SHAPE_128, k128_ranges(p)};
    else if (sh == SHAPE_256 && p.k >= 1024 && dma_k128_eligible(p)) plan = {KIND_DMA_K128, sh, 1};
    // (the same kernel on 128 x 128 tiles, where that is the shape and m, n, k are whole tiles
    // and blocks: 5 to 15 % over the 64-deep kernel of that shape; measured warm/cold, us:
    // 2048^3 14.6/15.1 -> 13.0/14.1, (1024, 3072, 3072) 17.1/23.2 -> 15.6/20.2,
    // (768, 4096, 2048) 12.3/12.9 -> 10.8/12.3, (256, 12544, 1152) 9.1/11.2 -> 8.3/10.4)
    else if (sh == SHAPE_128 && p.k >= 512 && dma_k128_eligible(p, true)) plan = {KIND_DMA_K128, sh, 1};
    // Aligned operands whose m or n is no multiple of the tile: the general forms of the same
    // kernel (loads redirected at the edges instead of padded operands), where the 64-deep
    // kernels with their masked edges used to serve.  On 256 x 256 tiles from k = 2048 on;
    // measured warm, us, overwriting: 4000^2 x 4096 105 -> 60, 4000^2 x 8192 193 -> 112,
    // 8000^2 x 4096 402 -> 254, (6000, 4000, 8192) 325 -> 198, (5008, 3008, 2048) 69 -> 42.
    else if (sh == SHAPE_256 && p.k >= 2048 && dma_k128_split_eligible(p, true))
      plan = {KIND_DMA_K128_SPLIT, SHAPE_256, 1};
    // On 128 x 128 tiles otherwise, from k = 768 on: 4000^2 x 1024 48 -> 30 (with an unsigned
    // operand 88 -> 33), 8000^2 x 1024 162 -> 93, (3000, 2000, 1024) 15.8 -> 14.0,
    // (3000, 2000, 4096) 45 -> 38, (1000, 3072, 768) 8.2 -> 6.7, (1000, 3072, 4096) 23 -> 21;
    // accumulating calls tie warm and gain cold ((3000, 2000, 1024) 19.7/25.7 -> 20.8/21.9).
    // Not at k = 512: (2048, 1568, 512) 6.6 -> 7.7.
    else if ((sh == SHAPE_256 || sh == SHAPE_128) && p.k >= 768 && dma_k128_split_eligible(p))
      plan = {KIND_DMA_K128_SPLIT, SHAPE_128, 1};
    // The same tiles one step below the count that makes 128 x 128 the shape above, on
    // problems with at least 1024 rows and columns and k from 2048: (1520, 1520, 2048)
    // 16.0/17.6 -> 13.3/14.3 us warm/cold, (1520, 1520, 8192) 56.5/56.0 -> 36.9/47.1.
    else if (p.k >= 2048 && p.m >= 1024 && p.n >= 1024 && tile_count(p, SHAPE_128) >= kComputeUnits / 2 &&
             tile_count(p, SHAPE_128) < 192 && dma_k128_split_eligible(p))
      plan = {KIND_DMA_K128_SPLIT, SHAPE_128, 1};
    else if (dma_eligible(p, sh)) plan = {KIND_DMA, sh, 1};
    // the register-staged kernel keeps its operands in flight in VGPRs, which a
    // 256 x 256 tile's accumulators leave no room for: it runs faster on 128 x 128
    // (and faster still on 128 x 64: its loads, 16 bytes at whatever alignment, are what
    // bounds it, and the narrower tile keeps more of them in flight per compute unit;
    // measured on 12 unaligned shapes from 1001 x 4099 x 513 to 4097 x 4099 x 2049: 9-25 % over
    // 128 x 128 on every one)
    // The wide side goes across the operand that is dearer to fetch again, a column-major A:
    // 8191 x 8193 x 8195 with such an A 4570 us on 128 x 64 tiles, 2570 on 64 x 128.
    else plan = {KIND_STAGED, sh == SHAPE_256 || sh == SHAPE_128 ? (p.a_sk == 1 ? SHAPE_128X64 : SHAPE_64X128) : sh, 1};
  }
  if (plan.kind == KIND_STAGED || plan.kind == KIND_DMA) {
    // float sums are not combined out of order: a float output splits k only through slots of
    // integer partial sums, which need room in a workspace
    const bool may_split = !p.out_float || (p.ws != nullptr && plan.kind == KIND_DMA);
    plan.splits = may_split ? forced_splits() : 1;
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
      // (an accumulating call needs no zero-fill launch and gains from two ranges already
      // at half a round of tiles: (128, 4096, 4096) 11.2 -> 8.8 us, overwriting 11.0 either way)
      // (a float output through slots needs no zeroed C either: it splits as an accumulating call does)
      if (((p.accumulate || p.out_float) ? tiles <= target / 2 : tiles < target / 2) && may_split) {
        const int64_t want = short_side <= 16 && small_tile ? (target + tiles - 1) / tiles : target / tiles;
        // the register-staged kernel has a shallow pipeline with little to amortise:
        // ranges of two k blocks already pay, and it tolerates twice the atomics
        const bool staged = plan.kind == KIND_STAGED;
        const int64_t shortest = staged ? 2 : 8;  // k blocks per range
        const int64_t most = nkt / shortest > 1 ? nkt / shortest : 1;
        const int64_t atomics_ok = (short_side <= 16 ? 64 : (short_side <= 64 ? 8 : 4)) * (staged ? 2 : 1);
        int64_t sp = want < most ? want : most;
        if (sp > atomics_ok) sp = atomics_ok;
        // the zero-fill launch of an overwriting call costs more than the ranges of a short k
        // save: (512, 512, 1024) 5.1 us whole, 6.4 us in two ranges (accumulating 5.0 and 4.5);
        // (512, 512, 2048) 6.7 and 7.3, (256, 256, 2048) 6.5 and 6.0, (512, 512, 4096) 10.6 and 8.7
        if (!p.accumulate && !p.out_float && short_side > 64 && p.k < (tiles <= 32 ? 2048 : 3072)) sp = 1;
        plan.splits = (int)sp;
      }
    }
  }
  return plan;
}

}  // namespace mip
