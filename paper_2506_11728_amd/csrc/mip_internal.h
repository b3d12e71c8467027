// Internal interface between the C-ABI layer and the HIP kernels.  Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mip {

// The problem after the host has normalised it: C is always row-major here (a
// column-major C is the row-major C^T = B^T A^T, so the host swaps the operand
// roles and flips their orders; paper Section 3, closing paragraph), and each
// 8-bit operand is described by two element strides, one of which is 1.
// Geometry of a convolution whose lowered matrix (paper Section 7.2: IM2COL) stands
// in for A: row i of A is output position (g, oy, ox) = i, its k index runs over
// (y, x, c) with c fastest, and A(i, (y, x, c)) is pixel (g, oy*stride + y - pad,
// ox*stride + x - pad, c) of the tensor at Problem::A, or 0 outside the image.
struct ConvGeom {
  int hi, wi, ci;  // image height, width, channels
  int wf;          // filter width (its height is k / (wf * ci))
  int ho, wo;      // output height, width
  int stride, pad;
};

struct Problem {
  int64_t m, n, k;
  const void *A;  // A(i,p) at A[i*a_sm + p*a_sk]
  int64_t a_sm, a_sk;
  const void *B;  // B(p,j) at B[p*b_sk + j*b_sn]
  int64_t b_sk, b_sn;
  int32_t *C;  // C(i,j) at C[i*ldc + j]
  int64_t ldc;
  int a_unsigned, b_unsigned;
  int accumulate;
  // 1: dequantised output (paper Section 7.3): C holds floats, float(sum) * scale
  // 2: requantised output: C holds int8 (ldc counts bytes), clip(rint(float(sum) * scale))
  int out_float;
  float scale;
  // batch > 1: that many independent problems of the same shape; problem z reads A + z*a_sb,
  // B + z*b_sb and writes C + z*c_sb (strides in elements).  Only the tile kernels, the
  // zero fill and the simple kernel take a batch (grid.z).
  int64_t batch = 1;
  int64_t a_sb = 0, b_sb = 0, c_sb = 0;
  // A and B are the library's own packed buffers: k-contiguous, and readable (with whatever
  // contents) up to the next multiple of 256 rows, so that whole tiles may be fetched
  bool rows_padded_to_256 = false;
  // device memory the kernels may use for the duration of the call (what is left of the
  // caller's workspace): slots of partial sums for split k (16-byte aligned)
  void *ws = nullptr;
  size_t ws_bytes = 0;
  // not null: the k sums of the signed operand of a product with one unsigned operand, one
  // int32 per column of B (a_unsigned) or row of A (b_unsigned), as pre-packed weights carry
  // them.  A kernel may use them in place of the sums it would accumulate, or ignore them.
  const int32_t *ksum = nullptr;
  // not null: A is never materialised, the kernel gathers it from the image tensor
  // (only the direct-to-LDS tile kernels can; a_sm is then the nominal row length k)
  const ConvGeom *conv = nullptr;
};

// Workgroup tile of the MFMA kernels (rows x columns of C).
enum Shape {
  SHAPE_256, SHAPE_128, SHAPE_64, SHAPE_64X256, SHAPE_256X64, SHAPE_64X128, SHAPE_128X64, SHAPE_COUNT
};

enum Kind {
  KIND_NONE = 0,  // nothing to launch (m == 0 or n == 0, or k == 0 with accumulate)
  KIND_FILL,      // k == 0, overwrite: C := 0
  KIND_SIMPLE,    // one thread per C element, any layout
  KIND_STAGED,    // MFMA tiles, operands staged through registers: any alignment, any size
  KIND_DMA,       // MFMA tiles, operands streamed global -> LDS directly (aligned, k % 64 == 0)
  KIND_DMA_K128,  // 256 x 256 (or, shape SHAPE_128, 128 x 128) tiles, 128-deep k blocks: large aligned problems
  KIND_DMA_K128_SPLIT,  // the same kernel, ragged edges allowed: 128 x 128 tiles with k cut into `splits` ranges, or (shape SHAPE_256) 256 x 256 tiles
  KIND_SLAB       // m <= 64: one workgroup per 16- or 32-column slab of B, all of k (splits = 1 or 2: slab width / 16)
};

struct Plan {
  Kind kind;
  Shape shape;  // KIND_STAGED and KIND_DMA
  int splits;   // k ranges worked on by separate workgroups (1 = no split)
};

Plan choose_plan(const Problem &p);
int64_t compute_units();  // of the current device, asked once (256 where no device answers)

// A kernel that takes more than 64 KB of dynamic LDS has to be told so once per device
// (hipFuncAttributeMaxDynamicSharedMemorySize); remembered, so that only the first launch of a
// kernel with a given size pays for the call.
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes);
const char *plan_name(const Plan &plan);  // static string

hipError_t launch_fill_zero(const Problem &p, hipStream_t s);
hipError_t launch_simple(const Problem &p, hipStream_t s);
hipError_t launch_staged(const Problem &p, Shape shape, int splits, hipStream_t s);

bool dma_k128_eligible(const Problem &p, bool small = false);  // small: its 128 x 128 form
// clocks: null, or room for two counters per workgroup (one per 256 x 256 tile, rounded up to a
// multiple of 8) that the kernel adds its shader clocks and 10 ns ticks to
hipError_t launch_dma_k128(const Problem &p, hipStream_t s, unsigned long long *clocks = nullptr,
                           bool small = false);

// The general 128 x 128 form of that kernel: any m and n (a strided operand's extent a multiple
// of 16), k in `splits` ranges that add into an int32 C (an overwriting call zeroes C first; a
// float or int8 output takes one range).
// large: on 256 x 256 tiles (one k range).
bool dma_k128_split_eligible(const Problem &p, bool large = false);
hipError_t launch_dma_k128_split(const Problem &p, int splits, hipStream_t s, bool large = false);

bool slab_eligible(const Problem &p, int nt);  // nt: slab width in blocks of 16 columns, 1 or 2
hipError_t launch_slab(const Problem &p, int nt, hipStream_t s);

#define MIP_DECLARE_DMA(BM, BN)                        \
  bool dma_eligible_##BM##x##BN(const Problem &p);     \
  hipError_t launch_dma_##BM##x##BN(const Problem &p, int splits, hipStream_t s);
MIP_DECLARE_DMA(256, 256)
MIP_DECLARE_DMA(128, 128)
MIP_DECLARE_DMA(64, 64)
MIP_DECLARE_DMA(64, 256)
MIP_DECLARE_DMA(256, 64)
MIP_DECLARE_DMA(64, 128)
MIP_DECLARE_DMA(128, 64)
#undef MIP_DECLARE_DMA

// The lowered matrix of a convolution written out: row n = (g, oy, ox) of M (pitch ldm
// bytes) holds the k = hf * wf * ci bytes that ConvGeom describes.
hipError_t launch_im2col(const ConvGeom &g, int64_t rows, int64_t k, const uint8_t *I, uint8_t *M,
                         int64_t ldm, hipStream_t s, int64_t kfill = 0);  // bytes k .. kfill - 1 zeroed

// The k x n matrix B (b_kc: already k-contiguous, pitch ldb; else row-major, pitch ldb)
// rewritten k-contiguous with pitch ldp; entries k .. kfill - 1 of every column are written
// as zeros (kfill <= k: nothing beyond k is written).
hipError_t launch_pack_b(int64_t k, int64_t n, const uint8_t *B, int64_t ldb, bool b_kc, uint8_t *P,
                         int64_t ldp, hipStream_t s, int64_t kfill = 0);

// sums[j] = the sum of the k bytes, read as signed 8-bit values, of column j of the
// k-contiguous matrix P (pitch ldp; 16 bytes at a time where k, ldp and P are multiples of 16).
hipError_t launch_column_sums(int64_t k, int64_t n, const uint8_t *P, int64_t ldp, int32_t *sums,
                              hipStream_t s);

// The convolution (p.conv set, image unsigned, filters k-contiguous with pitch k) with the
// augmented matrix gathered from image row segments staged in LDS: any channel count.
bool conv_rows_eligible(const Problem &p);
hipError_t launch_conv_rows(const Problem &p, hipStream_t s);

// Both operands of a GEMM packed in one launch: A (m rows of k, a_kc: k-contiguous with pitch
// lda, else k rows of m with pitch lda) to Ap and B (n columns of k, likewise) to Bp, both
// k-contiguous with pitch ldp, entries k .. kfill - 1 zeroed.
hipError_t launch_pack_pair(int64_t k, int64_t kfill, int64_t m, const uint8_t *A, int64_t lda,
                            bool a_kc, uint8_t *Ap, int64_t n, const uint8_t *B, int64_t ldb,
                            bool b_kc, uint8_t *Bp, int64_t ldp, hipStream_t s);

// 16-bit operands as byte planes (kernel_s16.hip).  X: rows x k int16, element (r, p) at
// X[r * s_r + p * s_k] with one stride 1; P: rows x 2 kp bytes, 16-byte aligned, kp a multiple
// of 16: per row the high bytes then the low bytes minus 128 (hi_first) or the other way
// round, zeros from p = k on.
hipError_t launch_split_planes(const int16_t *X, int64_t s_r, int64_t s_k, int64_t rows, int64_t k,
                               int64_t kp, uint8_t *P, bool hi_first, hipStream_t s);
// C = [C +] 65536 T1 + 256 T2 + T3 + the terms in the plane sums (see kernel_s16.hip); T1..T3
// dense m x n, C row-major with ldc.
// sA, sB: the byte sums of the plane matrices taken as 2 m (2 n) columns of kp bytes.
hipError_t launch_combine_planes(const int32_t *T1, const int32_t *T2, const int32_t *T3,
                                 const int32_t *sA, const int32_t *sB, int64_t m, int64_t n, int64_t k,
                                 int32_t *C, int64_t ldc, bool accumulate, hipStream_t s);

// `count` zeroed 32-bit counters in device memory that no other call in flight uses: the
// tickets of split k through partial-sum slots.  The kernels leave them zeroed.
hipError_t splitk_tickets(int64_t count, unsigned **out);

// Bytes of partial-sum slots the plan's split k wants (0: no split, or a kernel that adds
// into C with atomics whatever it is given).
size_t splitk_slot_bytes(const Problem &p, const Plan &plan);

bool dma_eligible(const Problem &p, Shape shape);
hipError_t launch_dma(const Problem &p, Shape shape, int splits, hipStream_t s);

}  // namespace mip
