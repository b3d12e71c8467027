/*
 * mipgemm: mixed-precision integer (MIP) GEMM for AMD MI355X (gfx950).
 *
 *     C (m x n, int32)  =  [ C + ]  A (m x k, 8-bit)  *  B (k x n, 8-bit)
 *
 * Every product of two 8-bit operands is formed exactly in 32 bits and summed
 * into a 32-bit accumulator (paper Section 5: inputs multiplied in INT8, result
 * accumulated in INT32; Section 3, figure "Reference GEMM algorithm": the
 * operation is C += A * B).  Sums wrap modulo 2^32; nothing saturates.  The
 * result is exact, so it does not depend on tile sizes or summation order.
 *
 * Storage (Section 3, closing paragraph: row- or column-major for all three
 * operands; Section 4 uses an explicit leading dimension ldC):
 *     MIPGEMM_ROW_MAJOR   X(r,c) = X[r*ld + c]   needs ld >= number of columns
 *     MIPGEMM_COL_MAJOR   X(r,c) = X[r + c*ld]   needs ld >= number of rows
 * Leading dimensions count elements, not bytes.  A transposed operand is the
 * same memory named with the other order.  No pointer or leading dimension
 * needs any alignment; alignment only decides how fast the operands load.
 *
 * Pointers.  A, B and C are DEVICE pointers owned by the caller.  The library
 * never allocates, frees or keeps them.  A and B are only read.  Only the
 * m x n elements of C are written: leading-dimension padding keeps its
 * contents.  With MIPGEMM_OVERWRITE the previous contents of C are never read.
 * C must not overlap A or B (not checked).  `stream` is a hipStream_t passed
 * as void* (NULL = the default stream).  `workspace` is device memory the call
 * may use until it completes on the stream.  For the GEMM entry points it is
 * optional (NULL / 0 is always accepted): with mipgemm_workspace_size() bytes,
 * 16-byte aligned, large products whose operands cannot be streamed as they are
 * stored (a pointer or leading dimension that is not a multiple of 16 bytes, k
 * not a multiple of 64) are first packed into it, k contiguous and padded with
 * zeros (the paper's Pack A / Pack B into aligned buffers A_c, B_c, Section
 * 4.1), and run several times faster; without it they run on slower kernels
 * that read the operands in place.  Results are the same bits either way.
 *
 * Execution.  Each call validates its arguments on the host, enqueues its
 * kernels on `stream` and returns without waiting.  Only kernels are enqueued
 * (no memory-set or copy operations), so a call may be recorded into a HIP
 * graph by stream capture and replayed.  Calls from several threads are safe:
 * the only state the library keeps is a table of kernels that have been granted
 * a large dynamic LDS size (guarded), the device's compute-unit count (read once)
 * and the tuning values below.
 *
 * Tuning values.  Four process-wide overrides exist for tests, tuning runs and
 * profiles; unset, the dispatcher decides.  They are taken from the environment
 * variables of the same names ONCE, at the first call into the library, and can
 * afterwards only be changed with mipgemm_set_tuning():
 *     MIPGEMM_VARIANT  kernel variant for the GEMM calls: "simple" (one thread per
 *                      element of C: a cross-check, hundreds of times slower),
 *                      "dma256k128", "dma128k128", "dma128k128split" (its general form: ragged
 *                      edges, k in MIPGEMM_SPLITK ranges), "slab16", "slab32", "slab64", "tile<shape>" or
 *                      "dma<shape>" with <shape> one of 256, 128, 64, 64x256,
 *                      256x64, 64x128, 128x64; a variant that cannot serve a
 *                      problem falls back (the names of mipgemm_variant_name say
 *                      what ran)
 *     MIPGEMM_SPLITK   number of k ranges of the tile kernels
 *     MIPGEMM_PACK     "always" / "never": the packed route whenever / never
 *     MIPGEMM_CONV     "im2col" / "rows": the convolution route
 *     MIPGEMM_STAGGER  10 ns ticks by which the tile rows of an XCD's patch start apart
 *                      in the kernel for large problems (tuning runs)
 *
 * Return value.  0 on success.  A negative value -i means that the i-th
 * argument (counted from 1 in the order of the prototype) is invalid: a
 * negative size, a null pointer for an operand that is not empty, a leading
 * dimension that is too small, an unknown order or mode, a size above
 * MIPGEMM_MAX_DIM, a null workspace with a non-zero workspace_bytes, or (in
 * the convolution entry points, which need theirs) a workspace that is too
 * small (reported on the workspace_bytes argument).  A positive value is the hipError_t of a failed
 * launch.  When a call fails validation nothing is enqueued and no memory is
 * touched.
 *
 * Empty problems.  m == 0 or n == 0: success, nothing is done.  k == 0: the sum
 * is empty, so MIPGEMM_OVERWRITE stores zeros and MIPGEMM_ACCUMULATE leaves C
 * as it is.
 */
#ifndef MIPGEMM_H
#define MIPGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIPGEMM_ROW_MAJOR 0
#define MIPGEMM_COL_MAJOR 1

#define MIPGEMM_OVERWRITE 0  /* C  = A * B */
#define MIPGEMM_ACCUMULATE 1 /* C += A * B */

/* largest m, n, k or leading dimension accepted */
#define MIPGEMM_MAX_DIM 2147483647LL

/* size of the static device buffer behind mipgemm_s8s8s32_noalloc, and the code that
 * call returns for a problem that would need more */
#define MIPGEMM_STATIC_SCRATCH_BYTES (64u << 20)
#define MIPGEMM_ERR_STATIC_SCRATCH (-100)

/*
 * Signed x signed: the paper's MIP GEMM proper (Section 5; every instruction it
 * surveys for this role, sdot / vmadot / the AMX tile product, takes two signed
 * 8-bit operands).  Argument numbers for error codes: m=1 n=2 k=3 A=4 lda=5
 * orderA=6 B=7 ldb=8 orderB=9 C=10 ldc=11 orderC=12 mode=13 workspace=14
 * workspace_bytes=15 stream=16.
 */
int mipgemm_s8s8s32(int64_t m, int64_t n, int64_t k,
                    const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB,
                    int32_t *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * mipgemm_s8s8s32 for callers that can neither allocate device memory nor bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments without the workspace pair (stream is argument
 * 14), same results, same errors.  Where mipgemm_s8s8s32 would pack its operands
 * into the caller's workspace, this call packs them into a static device buffer
 * of MIPGEMM_STATIC_SCRATCH_BYTES (64 MiB) that every GPU the library runs on
 * holds from the first such call until the process ends; the call allocates and
 * frees nothing.  A problem whose packed operands need more, i.e.
 * mipgemm_workspace_size-style (round_up(m, 256) + round_up(n, 256)) * kp bytes
 * above that limit, is rejected with MIPGEMM_ERR_STATIC_SCRATCH: nothing is
 * enqueued and nothing is touched (operands that are 16-byte aligned with k a
 * multiple of 64 are streamed as they are stored, need no buffer and have no such
 * limit).  All calls on one GPU share the one buffer: calls that overlap in time
 * on the same GPU (two streams, two threads) race on it and must be serialised by
 * the caller.  The buffer keeps the last call's contents; every byte a call reads
 * back it has written first, so nothing needs clearing.
 */
int mipgemm_s8s8s32_noalloc(int64_t m, int64_t n, int64_t k,
                            const int8_t *A, int64_t lda, int orderA,
                            const int8_t *B, int64_t ldb, int orderB,
                            int32_t *C, int64_t ldc, int orderC,
                            int mode,
                            void *stream);

/* MIPGEMM_STATIC_SCRATCH_BYTES as the loaded library was built with. */
size_t mipgemm_static_scratch_bytes(void);

/*
 * Unsigned A (for example activations quantized to 0..255) times signed B
 * (weights).  The uint8 values are taken at face value: no zero point is
 * subtracted (Section 7.3 describes a scale-only quantization).  Same
 * arguments, same numbering.
 */
int mipgemm_u8s8s32(int64_t m, int64_t n, int64_t k,
                    const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB,
                    int32_t *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * Signed A (weights) times unsigned B (activations): the operand roles of the
 * paper's convolution lowering, (m, n, k) = (c_o, b*h_o*w_o, c_i*h_f*w_f) with
 * the filters as A (Section 7.2).  Equal to mipgemm_u8s8s32 on the same memory
 * with A and B swapped and every order flipped (C^T = B^T A^T, Section 3).
 */
int mipgemm_s8u8s32(int64_t m, int64_t n, int64_t k,
                    const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB,
                    int32_t *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * A batch of independent signed x signed GEMMs of one shape in one call: problem
 * z = 0 .. batch-1 reads A + z*strideA and B + z*strideB and writes C + z*strideC
 * (strides in elements, >= 0; a stride of 0 shares that operand between the
 * problems; the C slices must not overlap, which is not checked).  This is the loop
 * over heads and sequences around the attention products of the paper's encoder
 * block (Section 7.2, the table of GEMM dimensions in the transformer encoder:
 * K^T Q and V E_1 for every head i and sequence j), made one launch, because
 * each of those products alone is far too small to occupy the device.  Everything
 * else is as for mipgemm_s8s8s32.  batch <= 65535; batch == 0 does nothing.
 * Argument numbers: m=1 n=2 k=3 A=4 lda=5 orderA=6 strideA=7 B=8 ldb=9 orderB=10
 * strideB=11 C=12 ldc=13 orderC=14 strideC=15 batch=16 mode=17 workspace=18
 * workspace_bytes=19 stream=20.
 */
int mipgemm_s8s8s32_batched(int64_t m, int64_t n, int64_t k,
                            const int8_t *A, int64_t lda, int orderA, int64_t strideA,
                            const int8_t *B, int64_t ldb, int orderB, int64_t strideB,
                            int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * The same strided batch with one unsigned operand, as mipgemm_u8s8s32 and
 * mipgemm_s8u8s32 are to mipgemm_s8s8s32 (Section 5.2 for the u8 x s8 pair): in the
 * encoder block the attention weights E_1 after the softmax are non-negative and
 * can be quantized to uint8 (Section 7.3 takes activations at face value), so
 * V E_1 per head is the s8 x u8 form.  Arguments, numbering, limits and errors
 * are those of mipgemm_s8s8s32_batched.
 */
int mipgemm_u8s8s32_batched(int64_t m, int64_t n, int64_t k,
                            const uint8_t *A, int64_t lda, int orderA, int64_t strideA,
                            const int8_t *B, int64_t ldb, int orderB, int64_t strideB,
                            int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

int mipgemm_s8u8s32_batched(int64_t m, int64_t n, int64_t k,
                            const int8_t *A, int64_t lda, int orderA, int64_t strideA,
                            const uint8_t *B, int64_t ldb, int orderB, int64_t strideB,
                            int32_t *C, int64_t ldc, int orderC, int64_t strideC,
                            int64_t batch, int mode,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * Dequantised output, the step the paper's quantization scheme puts right after
 * the integer GEMM (Section 7.3: C^r = s_A s_B A^q B^q = s_A s_B C^q): the same
 * three GEMMs, but C holds floats and receives
 *     overwrite:   C(i,j) = float(S(i,j)) * scale
 *     accumulate:  C(i,j) = fma(float(S(i,j)), scale, C(i,j))
 * where S(i,j) is the int32 sum of the s32 entry points (wrapping modulo 2^32),
 * float() rounds to nearest even, and `scale` is the product s_A * s_B formed
 * by the caller.  Each element is rounded at most twice: within 2^-23 relative
 * of the exact s_A s_B C^q.  The result does not depend on tile sizes: the sum
 * is completed in integers before anything is converted.  Same arguments, same
 * numbering and same rules as the s32 entry points; `scale` is argument 17 and
 * must be finite.
 */
int mipgemm_s8s8f32(int64_t m, int64_t n, int64_t k,
                    const int8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB,
                    float *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream, float scale);

int mipgemm_u8s8f32(int64_t m, int64_t n, int64_t k,
                    const uint8_t *A, int64_t lda, int orderA,
                    const int8_t *B, int64_t ldb, int orderB,
                    float *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream, float scale);

int mipgemm_s8u8f32(int64_t m, int64_t n, int64_t k,
                    const int8_t *A, int64_t lda, int orderA,
                    const uint8_t *B, int64_t ldb, int orderB,
                    float *C, int64_t ldc, int orderC,
                    int mode,
                    void *workspace, size_t workspace_bytes,
                    void *stream, float scale);

/*
 * Requantised output: the integer product brought back to 8 bits for the next
 * quantized layer.  The paper's scheme (Section 7.3) represents a real matrix X by
 * X^q with X ~ s_X X^q and gets C^r = s_A s_B C^q; in the output's own scale s_C
 * that is
 *     C(i,j) = clip( rint( float(S(i,j)) * scale ), -128, 127 ),  scale = s_A s_B / s_C
 * with S the int32 sum of the s32 entry points, float() and the product rounded to
 * nearest even in float32, rint rounding to the nearest integer with ties to even,
 * and saturation to the full int8 range (the paper does not spell this step out:
 * these are the readings taken).  C is int8 (ldc counts bytes; no alignment
 * needed), which makes the write a quarter of the int32 one: on shapes whose time
 * is the write of C (convolutions at large batch, short k) that is most of it.
 * Arguments and numbering as for the f32 entry points (`scale` = 17, finite);
 * `mode` must be MIPGEMM_OVERWRITE (a quantized output has no running sum: -13).
 * A problem with few tiles splits k only with workspace for slots of partial sums,
 * as the f32 entry points do (mipgemm_workspace_size_f32 bytes).
 */
int mipgemm_s8s8s8(int64_t m, int64_t n, int64_t k,
                   const int8_t *A, int64_t lda, int orderA,
                   const int8_t *B, int64_t ldb, int orderB,
                   int8_t *C, int64_t ldc, int orderC,
                   int mode,
                   void *workspace, size_t workspace_bytes,
                   void *stream, float scale);

int mipgemm_u8s8s8(int64_t m, int64_t n, int64_t k,
                   const uint8_t *A, int64_t lda, int orderA,
                   const int8_t *B, int64_t ldb, int orderB,
                   int8_t *C, int64_t ldc, int orderC,
                   int mode,
                   void *workspace, size_t workspace_bytes,
                   void *stream, float scale);

int mipgemm_s8u8s8(int64_t m, int64_t n, int64_t k,
                   const int8_t *A, int64_t lda, int orderA,
                   const uint8_t *B, int64_t ldb, int orderB,
                   int8_t *C, int64_t ldc, int orderC,
                   int mode,
                   void *workspace, size_t workspace_bytes,
                   void *stream, float scale);

/*
 * Convolution by lowering (paper Section 7.2: O = CONV(F, I); the input tensor is
 * turned into an augmented matrix by IM2COL and the convolution into a GEMM of
 * dimensions (m, n, k) = (c_o, b h_o w_o, c_i h_f w_f); the paper counts the
 * transform in its GEMM times).
 *
 * Tensors are dense, innermost index last, in the order the paper gives their
 * sizes: I is b x h_i x w_i x c_i (uint8 activations, taken at face value), F is
 * c_o x h_f x w_f x c_i (int8), O is b x h_o x w_o x c_o (int32), with
 * h_o = (h_i + 2 pad - h_f) / stride + 1 (integer division) and w_o likewise.
 *     O(g, oy, ox, o) [+]= sum over (y, x, c) of
 *                          F(o, y, x, c) * I(g, oy*stride + y - pad, ox*stride + x - pad, c)
 * where positions outside the image contribute nothing (zero padding); the
 * filter is not flipped; sums wrap modulo 2^32 as in the GEMM.  As a GEMM, F is A
 * (c_o x k, row-major), the augmented matrix is B (k x n, k contiguous) and O is
 * C (column-major with ldc = c_o), k index (y, x, c) with c fastest, n index
 * (g, oy, ox) with ox fastest.
 *
 * mipgemm_conv_s8u8s32 gathers the augmented matrix on the fly inside the
 * multiplying kernel, so that nothing is written but O and no workspace is
 * needed, in two cases: c_i a multiple of 64 with F and I 16-byte aligned (the
 * GEMM tile kernels take their operand addresses from the image), and any c_i
 * with a short k (up to about 600, e.g. the 3-channel 7 x 7 first layer of a
 * network: a kernel that stages image row segments on chip).  Otherwise it
 * writes the augmented matrix into `workspace` first
 * (mipgemm_conv_workspace_size bytes; rows padded with zeros to whole k blocks,
 * the filters re-pitched the same way behind it) and multiplies the two.  Pointers are device pointers owned by the caller;
 * same execution and error conventions as the GEMM entry points.  Argument
 * numbers: b=1 hi=2 wi=3 ci=4 co=5 hf=6 wf=7 stride=8 pad=9 F=10 I=11 O=12 mode=13
 * workspace=14 workspace_bytes=15 stream=16.  Sizes must be positive (b and c_o may
 * be 0: nothing is done), the filter must fit the padded image, and b*h_i*w_i*c_i,
 * b*h_o*w_o and c_i*h_f*w_f must stay below 2^31.
 */
int mipgemm_conv_s8u8s32(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                         int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                         const int8_t *F, const uint8_t *I, int32_t *O,
                         int mode,
                         void *workspace, size_t workspace_bytes,
                         void *stream);

/*
 * The same convolution with a float O and the dequantising scale of Section 7.3
 * fused into the write-back, exactly as in the f32 GEMM entry points:
 * overwrite O = float(S) * scale, accumulate O = fma(float(S), scale, O), with S
 * the int32 sum above, completed in integers before anything is converted.
 * `scale` is argument 17 and must be finite.
 */
int mipgemm_conv_s8u8f32(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                         int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                         const int8_t *F, const uint8_t *I, float *O,
                         int mode,
                         void *workspace, size_t workspace_bytes,
                         void *stream, float scale);

/*
 * The same convolutions with the k-sums of the filters supplied (Section 4.1 carried to
 * constant weights, as mipgemm_pack_weights does for a GEMM): the image is unsigned, the
 * matrix instructions are signed, so the kernels multiply `pixel - 128` and add
 * 128 * sum over k of F(o, k) per filter o; without the sums every call adds the filter
 * fragments up again as they pass through the registers.  mipgemm_conv_filter_sums
 * computes sums[o] (DEVICE memory, c_o int32) from the filter tensor, k = h_f w_f c_i, once;
 * argument numbers co=1 k=2 F=3 sums=4 stream=5.  The *_with_sums calls take it as their
 * last argument (number 17 for the s32 form, 18 for the f32 form; must not be null) and
 * give the same results as the plain calls; the kernels that gather through the tile
 * kernels and the written-out route use the sums, the row-segment kernel computes its own.
 */
int mipgemm_conv_filter_sums(int64_t co, int64_t k, const int8_t *F, int32_t *sums, void *stream);
int mipgemm_conv_s8u8s32_with_sums(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                   int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                                   const int8_t *F, const uint8_t *I, int32_t *O,
                                   int mode,
                                   void *workspace, size_t workspace_bytes,
                                   void *stream, const int32_t *filter_sums);
int mipgemm_conv_s8u8f32_with_sums(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                   int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                                   const int8_t *F, const uint8_t *I, float *O,
                                   int mode,
                                   void *workspace, size_t workspace_bytes,
                                   void *stream, float scale, const int32_t *filter_sums);

/*
 * The convolution with an int8 output requantised for the next quantized layer, as
 * mipgemm_s8u8s8 does for a GEMM: O(g, oy, ox, o) = clip(rint(scale * sum), -128, 127),
 * the sum converted to float32, one float32 multiplication, ties to even, O a tensor
 * of b x h_o x w_o x c_o BYTES.  At large batch most layers are bound by the write of
 * their output, which this form cuts to a quarter.  `mode` must be MIPGEMM_OVERWRITE
 * (-13); `scale` (argument 17) must be finite; `filter_sums` (argument 18) is the result
 * of mipgemm_conv_filter_sums or NULL.  Workspace as for mipgemm_conv_s8u8s32.
 */
int mipgemm_conv_s8u8s8(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                        int64_t co, int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                        const int8_t *F, const uint8_t *I, int8_t *O,
                        int mode,
                        void *workspace, size_t workspace_bytes,
                        void *stream, float scale, const int32_t *filter_sums);

/*
 * Bytes of workspace mipgemm_conv_s8u8s32 / mipgemm_conv_s8u8f32 need for these sizes when its pointers
 * are 16-byte aligned: 0 when the augmented matrix is gathered on the fly (see
 * above), else room for it.  Returns 0 for invalid sizes.
 */
size_t mipgemm_conv_workspace_size(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                   int64_t co, int64_t hf, int64_t wf,
                                   int64_t stride, int64_t pad);

/*
 * The same for a call whose F or I is NOT 16-byte aligned: the tile kernels cannot
 * gather from such tensors, so layers that need no workspace above may need one
 * here (a call without it fails with -14 or -15 and touches nothing).
 */
size_t mipgemm_conv_workspace_size_unaligned(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                             int64_t co, int64_t hf, int64_t wf,
                                             int64_t stride, int64_t pad);

/*
 * The augmented matrix alone (IM2COL of Section 7.2): M has one row per output
 * position n = (g, oy, ox) and k = h_f w_f c_i bytes per row, rows `ldm` bytes apart
 * (ldm >= k); bytes of a row beyond k are not written.  As the B operand of a
 * GEMM it is k x n, column-major, ldb = ldm.  Argument numbers: b=1 hi=2 wi=3
 * ci=4 hf=5 wf=6 stride=7 pad=8 I=9 M=10 ldm=11 stream=12.
 */
int mipgemm_im2col_u8(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                      int64_t hf, int64_t wf, int64_t stride, int64_t pad,
                      const uint8_t *I, uint8_t *M, int64_t ldm,
                      void *stream);

/*
 * Name of the path mipgemm_conv_s8u8s32 takes for these sizes with 16-byte
 * aligned pointers: "implicit:<kernel variant>" or "im2col+<kernel variant>".
 * Host-only; for tests and benchmarks.  Returns a static string.
 */
const char *mipgemm_conv_variant_name(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                                      int64_t co, int64_t hf, int64_t wf,
                                      int64_t stride, int64_t pad);

/*
 * Weight pre-packing (paper Section 4.1: B is packed into a buffer that the
 * micro-kernel reads with unit stride, at a cost amortised over its reuse; for
 * inference the weights are constant, so the packing can be done once, ahead of
 * time).  Rewrites the k x n 8-bit matrix B, stored in either order, with k
 * contiguous: P(p, j) = P[p + j*ldp], ldp >= k, i.e. the same matrix in
 * MIPGEMM_COL_MAJOR order with ldb = ldp, which is how P is then passed as the B
 * of the GEMM entry points.  The GEMMs accept either order directly; packing pays
 * when a few rows of A (m <= 16) meet the same B many times, because the skinny-m
 * kernel streams a k-contiguous B in whole cache-line runs.  Bytes of P beyond the
 * k entries of a column are not written; B and P must not overlap (not checked);
 * signedness does not matter (bytes are moved).  Argument numbers: k=1 n=2 B=3
 * ldb=4 orderB=5 P=6 ldp=7 stream=8.
 */
int mipgemm_pack_b(int64_t k, int64_t n,
                   const void *B, int64_t ldb, int orderB,
                   void *P, int64_t ldp,
                   void *stream);

/*
 * C (+)= A B with 16-bit operands, int16 x int16 -> int32: the (i32, i16, i16) forms of
 * the paper's table of matrix-oriented instructions (vpdpwssd, smopa).  This device has no
 * integer matrix instruction for 16-bit operands, so the product is built from 8-bit ones:
 * with x' = x - 128 every int16 is two signed bytes, x' = 256 h + l, and the sum over k of
 * a b is 65536 (ah bh) + 256 (ah bl + al bh) + (al bl) + 128 (sum a' + sum b') + 16384 k,
 * three s8 x s8 GEMMs of this library on the byte planes (the middle one of depth 2 k) and
 * one pass that puts the pieces together: about four times the work of an 8-bit product of
 * the same size.  Sums wrap modulo 2^32, which products of up to 2^30 reach much sooner
 * than bytes do.  Arguments and their numbers as for mipgemm_s8s8s32 (lda, ldb count
 * elements); the workspace is REQUIRED here for k > 0: mipgemm_workspace_size_s16(m, n, k)
 * bytes of device memory (planes, plane sums, three m x n int32 products); a null
 * workspace is -14, one that is too small -15, and nothing is touched.
 */
size_t mipgemm_workspace_size_s16(int64_t m, int64_t n, int64_t k);
int mipgemm_s16s16s32(int64_t m, int64_t n, int64_t k,
                      const int16_t *A, int64_t lda, int orderA,
                      const int16_t *B, int64_t ldb, int orderB,
                      int32_t *C, int64_t ldc, int orderC,
                      int mode,
                      void *workspace, size_t workspace_bytes,
                      void *stream);

/*
 * Pre-packed weights as an object of their own (Section 4.1 carried to constant
 * weights: everything that depends on B alone is done once): the k x n signed
 * matrix B, stored in either order, rewritten into `packed` as
 *   - its columns with k contiguous, each padded with zeros to kp bytes (k rounded
 *     up to a multiple of 128, of 64 when k < 1024; at least one such block), the
 *     column count padded with zero columns to a multiple of 256 (at least 256), so
 *     that every kernel may fetch whole blocks and whole tiles of it, then
 *   - n int32 k-sums, s(j) = sum over p of B(p, j) (wrapping modulo 2^32): what a
 *     product with unsigned activations needs of B beside the product itself,
 *     sum_p a b = sum_p (a - 128) b + 128 s, the matrix instructions being signed.
 *     Without them every call sums the fragments of B again as they pass through
 *     the registers, which costs 12 to 25 % of the time of a large u8 x s8 product.
 * mipgemm_packed_weights_bytes(k, n) is the size of that object (0 for invalid
 * sizes); `packed` is DEVICE memory of at least that size, 16-byte aligned, owned
 * by the caller, and must not overlap B.  Three small launches on `stream`.
 * Argument numbers: k=1 n=2 B=3 ldb=4 orderB=5 packed=6 packed_bytes=7 stream=8.
 */
size_t mipgemm_packed_weights_bytes(int64_t k, int64_t n);
int mipgemm_pack_weights(int64_t k, int64_t n,
                         const int8_t *B, int64_t ldb, int orderB,
                         void *packed, size_t packed_bytes,
                         void *stream);

/*
 * C (+)= A B with B given as packed weights (mipgemm_pack_weights with the same k and
 * n): mipgemm_s8s8s32 / mipgemm_u8s8s32 with `packed` in the place of B, ldb and
 * orderB.  Same results, bit for bit, as the calls on the unpacked matrix; the
 * unsigned form takes the k-sums from the packed object where the kernel it is
 * dispatched to can use them (the direct-to-LDS tile kernels on an unsplit k) and
 * computes them as usual elsewhere.  Everything else (orders of A and C, mode,
 * workspace, stream, errors) as in mipgemm_s8s8s32.  Argument numbers: m=1 n=2 k=3
 * A=4 lda=5 orderA=6 packed=7 C=8 ldc=9 orderC=10 mode=11 workspace=12
 * workspace_bytes=13 stream=14.
 */
int mipgemm_s8s8s32_packed(int64_t m, int64_t n, int64_t k,
                           const int8_t *A, int64_t lda, int orderA,
                           const void *packed,
                           int32_t *C, int64_t ldc, int orderC,
                           int mode,
                           void *workspace, size_t workspace_bytes,
                           void *stream);
int mipgemm_u8s8s32_packed(int64_t m, int64_t n, int64_t k,
                           const uint8_t *A, int64_t lda, int orderA,
                           const void *packed,
                           int32_t *C, int64_t ldc, int orderC,
                           int mode,
                           void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Bytes of device workspace with which a GEMM call of these sizes and orders
 * takes the packed route (see "Pointers" above), taking the tightest leading
 * dimensions and 16-byte aligned pointers: 0 when such operands are streamed as
 * they are, when the shape is one for which packing does not pay (m or n below
 * 96, k below 192, m*n*k below 2^22), and for invalid sizes.  Operands with other leading
 * dimensions or pointers need (round_up(m, 256) + round_up(n, 256)) * kp bytes,
 * kp = k rounded up to a multiple of 128 (of 64 when k < 1024); a call uses the packed route whenever
 * it would pay and the workspace it is given is that large.
 */
size_t mipgemm_workspace_size(int64_t m, int64_t n, int64_t k,
                              int orderA, int orderB, int orderC);

/*
 * The same for the f32 entry points.  Besides the packed operands, a float-output
 * call can use room for slots of partial sums: a problem with too few tiles of C
 * to occupy the device splits k over several workgroups per tile, and since float
 * sums must not be combined in arbitrary order, the workgroups of a tile meet in
 * such slots with their int32 partial sums (splits x tile size x 4 bytes per tile;
 * the last to arrive adds them up, still in integers, and converts once: same
 * result as an unsplit call).  Without the room such a call keeps all of k in one
 * workgroup per tile and runs up to twice as long on long-k, few-tile shapes.
 * (The per-tile counters of that scheme live in a 4 MiB static device array of
 * the library, handed out in rotation, so that concurrent calls use different
 * ones; the int32 entry points add their k ranges into C with atomics and need
 * no slots.)
 */
size_t mipgemm_workspace_size_f32(int64_t m, int64_t n, int64_t k,
                                  int orderA, int orderB, int orderC);

/*
 * Static, human-readable text for a return value of the functions above.  For a
 * negative code the text gives the argument number and, in parentheses, the name
 * that argument has in the GEMM entry points (the convolution entry points number
 * their own arguments as their comments say).
 */
const char *mipgemm_strerror(int code);

/*
 * Name of the kernel variant the dispatcher picks for these sizes, orders,
 * leading dimensions and pointer alignments (all pointers taken as 16-byte
 * aligned when `aligned16` is non-zero), for an overwriting call without workspace
 * (an accumulating call into an int32 C may take tiles with split k where this
 * names the skinny-m kernel).  Host-only, launches nothing; meant for tests,
 * benchmarks and profiles.  Returns a static string.
 */
const char *mipgemm_variant_name(int64_t m, int64_t n, int64_t k,
                                 int64_t lda, int orderA,
                                 int64_t ldb, int orderB,
                                 int64_t ldc, int orderC,
                                 int a_unsigned, int b_unsigned, int aligned16);

/*
 * The same with the call's mode (MIPGEMM_OVERWRITE or MIPGEMM_ACCUMULATE) taken into
 * account: mode is argument 13 here.
 */
const char *mipgemm_variant_name_for_mode(int64_t m, int64_t n, int64_t k,
                                          int64_t lda, int orderA,
                                          int64_t ldb, int orderB,
                                          int64_t ldc, int orderC,
                                          int a_unsigned, int b_unsigned, int aligned16,
                                          int mode);

/*
 * Sets one tuning value (see "Tuning values" above) for the whole process: `name`
 * is the variable's name, `value` its text as in the environment, NULL or "" to
 * clear it.  Returns 0, or -1 for an unknown name or a value that does not parse
 * (nothing changes then).  Calls already running keep the values they started with;
 * meant for tests and tuning scripts, not for steering concurrent production calls.
 */
int mipgemm_set_tuning(const char *name, const char *value);

/*
 * The same for a call that is given a workspace of sufficient size: "packed+"
 * and the kernel that multiplies the packed operands when the packed route is
 * taken, else what mipgemm_variant_name returns.
 */
const char *mipgemm_variant_name_with_workspace(int64_t m, int64_t n, int64_t k,
                                                int64_t lda, int orderA,
                                                int64_t ldb, int orderB,
                                                int64_t ldc, int orderC,
                                                int a_unsigned, int b_unsigned, int aligned16);

/*
 * Device characterisation for benchmarks: the throughput, in 10^12 operations
 * per second (2 operations per multiply-accumulate, the count of the paper's
 * Section 7.4), of the int8 matrix instruction the GEMM kernels are built on
 * when every operand is already in registers.  No kernel that uses the
 * instruction can exceed it on this device at this moment.  pattern 0 uses
 * operands that are almost all zero bits; pattern 1 uses random bytes that
 * change every iteration, as a GEMM on random data does.  The device is
 * power-limited, so the two differ widely.  One iteration is 128 x 128 x 64
 * multiply-accumulates per wave.  `tops` is a HOST pointer.  Unlike the GEMM
 * entry points this call allocates a few bytes of device memory, waits for its
 * kernel to finish and frees them again.  Returns 0, the negative number of an
 * invalid argument (1 pattern, 2 iterations, 4 tops), or a positive hipError_t.
 * (The rate of pattern 1 includes register moves between the matrix
 * instructions; mipgemm_mfma_ceiling_clocked has patterns without them.)
 */
int mipgemm_mfma_ceiling(int pattern, int iterations, void *stream, double *tops);

/*
 * The same with more operand patterns and the shader clock the device ran at while
 * the loop was executing (each workgroup reads the shader clock counter and the
 * constant 100 MHz counter before and after its loop; `shader_mhz`, a HOST
 * pointer, may be NULL).  pattern 0 and 1 as above; in pattern 1 the operands are
 * rotated in registers between iterations, which puts 128 register moves between
 * the 32 matrix instructions of an iteration.  pattern 2: random bytes in two fixed
 * operand sets used in turn; pattern 3: random bytes in six fixed operand sets used
 * in turn; in both the loop holds nothing but matrix instructions.  Patterns 0 to 3
 * run v_mfma_i32_32x32x32_i8; pattern 4 (near-zero constants) and pattern 5 (random
 * bytes, one fixed operand set) run v_mfma_i32_16x16x64_i8, the instruction of the
 * kernel for large problems, on the same 128 x 128 block per wave.
 */
int mipgemm_mfma_ceiling_clocked(int pattern, int iterations, void *stream,
                                 double *tops, double *shader_mhz);

/*
 * For benchmarks: mipgemm_s8s8s32 on the kernel for large aligned problems (256 x
 * 256 tiles, 128-deep k blocks), with every workgroup adding the shader clocks and
 * the 10 ns ticks of its main loop to clocks[2 w] and clocks[2 w + 1] (w = the
 * workgroup's number; `clocks` is DEVICE memory that the caller has zeroed, two
 * 64-bit counters per tile of C with the tile count rounded up to a multiple of 8,
 * `clocks_bytes` its size).  Sum of clocks / sum of ticks * 100 = shader MHz.
 * Arguments 1..13 as in mipgemm_s8s8s32, then stream=14 clocks=15 clocks_bytes=16.
 * Returns -1 when the problem is not one that kernel takes (m, n multiples of 256,
 * k a multiple of 128, 16-byte aligned operands).
 */
int mipgemm_s8s8s32_clocked(int64_t m, int64_t n, int64_t k,
                            const int8_t *A, int64_t lda, int orderA,
                            const int8_t *B, int64_t ldb, int orderB,
                            int32_t *C, int64_t ldc, int orderC,
                            int mode, void *stream,
                            unsigned long long *clocks, size_t clocks_bytes);

#ifdef __cplusplus
}
#endif
#endif /* MIPGEMM_H */
