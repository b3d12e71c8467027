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
 * may use until it completes on the stream; pass at least
 * mipgemm_workspace_size() bytes, or NULL / 0 when that size is 0.
 *
 * Execution.  Each call validates its arguments on the host, enqueues its
 * kernels on `stream` and returns without waiting.  The library holds no
 * mutable global state: calls from several threads are safe.
 *
 * Return value.  0 on success.  A negative value -i means that the i-th
 * argument (counted from 1 in the order of the prototype) is invalid: a
 * negative size, a null pointer for an operand that is not empty, a leading
 * dimension that is too small, an unknown order or mode, a size above
 * MIPGEMM_MAX_DIM, or a workspace that is too small (reported on the
 * workspace_bytes argument).  A positive value is the hipError_t of a failed
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
 * Bytes of device workspace a call with these sizes and orders may use.
 * Returns 0 when none is needed (and for invalid sizes).
 */
size_t mipgemm_workspace_size(int64_t m, int64_t n, int64_t k,
                              int orderA, int orderB, int orderC);

/* Static, human-readable text for a return value of the functions above. */
const char *mipgemm_strerror(int code);

/*
 * Name of the kernel variant the dispatcher picks for these sizes, orders,
 * leading dimensions and pointer alignments (all pointers taken as 16-byte
 * aligned when `aligned16` is non-zero).  Host-only, launches nothing; meant
 * for tests, benchmarks and profiles.  Returns a static string.
 */
const char *mipgemm_variant_name(int64_t m, int64_t n, int64_t k,
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
 */
int mipgemm_mfma_ceiling(int pattern, int iterations, void *stream, double *tops);

#ifdef __cplusplus
}
#endif
#endif /* MIPGEMM_H */
