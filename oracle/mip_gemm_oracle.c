/*
 * CPU oracle for the mixed-precision integer (MIP) GEMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is
 * compared against; the product never calls it, links it or falls back to it.
 * It shares no code, header, table or helper with the HIP path.
 *
 * What it computes (paper, abstract and Section 5 "Micro-kernel for
 * DOT-oriented SIMD units and MIP": inputs multiplied in INT8, result
 * accumulated in INT32; Section 3, Figure "Reference GEMM algorithm":
 * C += A * B):
 *
 *     for 0 <= i < m, 0 <= j < n:
 *         S(i,j) = sum_{p=0}^{k-1} (int32) A(i,p) * (int32) B(p,j)
 *         C(i,j) = S(i,j)            (overwrite)
 *         C(i,j) = C(i,j) + S(i,j)   (accumulate)
 *
 * The paper's blocked algorithm is a reordering of this sum, and integer
 * addition is associative, so the method reaches exactly this definition; the
 * oracle is therefore the definition written out as three plain loops, with no
 * blocking, packing or reordering.
 *
 * Readings where the paper is silent:
 *   - int32 overflow: two's-complement wraparound (arithmetic modulo 2^32),
 *     done here in uint32_t so that C leaves no behaviour undefined.
 *   - every int8 product is exact in int32 (no int16 intermediate as in the
 *     ARMv8.0 kernel of Section 5.1, which is an artefact of that ISA).
 *   - a uint8 operand is taken at face value, 0..255 (Section 7.3 describes a
 *     scale-only quantization scheme: no zero point is subtracted).
 *   - m == 0 or n == 0: nothing is touched.  k == 0: the sum is empty, so
 *     overwrite stores 0 and accumulate leaves C as it is.
 *
 * Storage (Section 3, last paragraph: row- or column-major for all three
 * operands, explicit leading dimension as in the ldC of Section 4):
 *     row-major    X(r,c) = X[r*ld + c]
 *     column-major X(r,c) = X[r + c*ld]
 * ld is counted in elements.  Elements of C outside the m x n matrix (the
 * leading-dimension padding) are never written.
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force int64 dot products,
 * exhaustive 1x1x1 over all byte pairs, constant-matrix closed forms,
 * identity / permutation matrices, row and column sums, linearity and k-split,
 * layout identities, the u8 <-> s8 identity, numpy int64 matmul, the
 * instruction-tile definitions the paper prints (sdot, vmadot, AMX tile) and a
 * hand-worked example stored under tests/golden/.  The dequantised variant at
 * the end of the file is pinned by the same hand-worked example with exact
 * scales, by scale = 1 against the integer function, by closed forms and by
 * linearity in the scale.  The requantised variant is pinned by hand-worked
 * values (scale 1/8 of the same example, a row of exact ties and saturating
 * values, and a sum above 2^24 whose float32 image decides the tie), by scale = 1
 * on small sums against the integer function, by the fp64 dequantised function
 * away from ties, and by the same three IEEE operations done by numpy.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

enum { ORACLE_ROW_MAJOR = 0, ORACLE_COL_MAJOR = 1 };
enum { ORACLE_OVERWRITE = 0, ORACLE_ACCUMULATE = 1 };

/* position of X(r,c) in its buffer */
static size_t at(int64_t r, int64_t c, int64_t ld, int order)
{
    if (order == ORACLE_ROW_MAJOR)
        return (size_t)r * (size_t)ld + (size_t)c;
    return (size_t)r + (size_t)c * (size_t)ld;
}

/* one byte read as int8 or as uint8, widened to 32 bits before any multiply */
static uint32_t widen(const void *X, size_t pos, int is_unsigned)
{
    if (is_unsigned)
        return (uint32_t)((const uint8_t *)X)[pos];
    return (uint32_t)(int32_t)((const int8_t *)X)[pos];
}

/*
 * Returns 0, or -1 when an argument is malformed (negative size, leading
 * dimension too small, unknown order or mode).  Host pointers only.
 */
int oracle_mip_gemm(int a_unsigned, int b_unsigned,
                    int64_t m, int64_t n, int64_t k,
                    const void *A, int64_t lda, int orderA,
                    const void *B, int64_t ldb, int orderB,
                    int32_t *C, int64_t ldc, int orderC,
                    int mode)
{
    if (m < 0 || n < 0 || k < 0) return -1;
    if (orderA != ORACLE_ROW_MAJOR && orderA != ORACLE_COL_MAJOR) return -1;
    if (orderB != ORACLE_ROW_MAJOR && orderB != ORACLE_COL_MAJOR) return -1;
    if (orderC != ORACLE_ROW_MAJOR && orderC != ORACLE_COL_MAJOR) return -1;
    if (mode != ORACLE_OVERWRITE && mode != ORACLE_ACCUMULATE) return -1;
    if (lda < (orderA == ORACLE_ROW_MAJOR ? k : m)) return -1;
    if (ldb < (orderB == ORACLE_ROW_MAJOR ? n : k)) return -1;
    if (ldc < (orderC == ORACLE_ROW_MAJOR ? n : m)) return -1;

    uint32_t *Cu = (uint32_t *)C;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        if (mode == ORACLE_OVERWRITE)
            for (int64_t j = 0; j < n; ++j)
                Cu[at(i, j, ldc, orderC)] = 0u;
        for (int64_t p = 0; p < k; ++p) {
            uint32_t a = widen(A, at(i, p, lda, orderA), a_unsigned);
            for (int64_t j = 0; j < n; ++j) {
                uint32_t b = widen(B, at(p, j, ldb, orderB), b_unsigned);
                Cu[at(i, j, ldc, orderC)] += a * b;
            }
        }
    }
    return 0;
}

/*
 * Dequantised result, fp64: the step the paper's quantization scheme applies to
 * the integer product (Section 7.3: C^r = s_A s_B A^q B^q = s_A s_B C^q).
 *
 *     out(i,j) = scale * S(i,j)                 (overwrite)
 *     out(i,j) = C0(i,j) + scale * S(i,j)       (accumulate)
 *
 * S is the int32 sum defined at the top of this file (same wraparound reading),
 * `scale` the product s_A * s_B handed over as a float, C0 the float matrix the
 * caller wants updated (read through ldc / orderC, may be NULL for overwrite).
 * The arithmetic after the integer sum is done in double: every int32 and every
 * float is exact in double, so scale * S is exact and the one addition is
 * rounded once, far below the float result it is compared with.
 * `out` is a dense row-major m x n array of doubles.
 */
int oracle_mip_gemm_dequant(int a_unsigned, int b_unsigned,
                            int64_t m, int64_t n, int64_t k,
                            const void *A, int64_t lda, int orderA,
                            const void *B, int64_t ldb, int orderB,
                            float scale,
                            const float *C0, int64_t ldc, int orderC,
                            int mode, double *out)
{
    if (m < 0 || n < 0 || k < 0) return -1;
    if (orderA != ORACLE_ROW_MAJOR && orderA != ORACLE_COL_MAJOR) return -1;
    if (orderB != ORACLE_ROW_MAJOR && orderB != ORACLE_COL_MAJOR) return -1;
    if (orderC != ORACLE_ROW_MAJOR && orderC != ORACLE_COL_MAJOR) return -1;
    if (mode != ORACLE_OVERWRITE && mode != ORACLE_ACCUMULATE) return -1;
    if (lda < (orderA == ORACLE_ROW_MAJOR ? k : m)) return -1;
    if (ldb < (orderB == ORACLE_ROW_MAJOR ? n : k)) return -1;
    if (ldc < (orderC == ORACLE_ROW_MAJOR ? n : m)) return -1;
    if (mode == ORACLE_ACCUMULATE && !C0 && m > 0 && n > 0) return -1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            uint32_t s = 0u;
            for (int64_t p = 0; p < k; ++p)
                s += widen(A, at(i, p, lda, orderA), a_unsigned)
                   * widen(B, at(p, j, ldb, orderB), b_unsigned);
            double r = (double)scale * (double)(int32_t)s;
            if (mode == ORACLE_ACCUMULATE)
                r += (double)C0[at(i, j, ldc, orderC)];
            out[(size_t)i * (size_t)n + (size_t)j] = r;
        }
    }
    return 0;
}

/*
 * Requantised result, int8: the integer product brought back to 8 bits for the
 * next quantized layer.  The paper's scheme (Section 7.3) represents a real
 * matrix X by X^q with X ~ s_X X^q (symmetric, scale only); the product
 * C^r = s_A s_B C^q expressed in the output's own scale s_C is therefore
 *
 *     Q(i,j) = clip( rint( scale * S(i,j) ), -128, 127 ),   scale = s_A s_B / s_C
 *
 * The paper does not spell this step out.  Readings taken (both the oracle and
 * the GPU take the rounding decision in the same precision, float32, which is
 * the precision the GPU entry point computes in):
 *   - S is the int32 sum defined at the top of this file (wraparound reading);
 *   - S is converted to float32 (round to nearest, ties to even), multiplied by
 *     `scale` in one float32 multiplication, and rounded to an integer with
 *     ties to even (rintf in the default rounding mode);
 *   - the result saturates to the full int8 range [-128, 127];
 *   - there is no accumulate form (a quantized output has no running sum);
 *   - `scale` must be finite.
 * Q is m x n int8 with leading dimension ldq in order orderQ; bytes outside the
 * m x n matrix are never written.
 */
int oracle_mip_gemm_requant(int a_unsigned, int b_unsigned,
                            int64_t m, int64_t n, int64_t k,
                            const void *A, int64_t lda, int orderA,
                            const void *B, int64_t ldb, int orderB,
                            float scale,
                            int8_t *Q, int64_t ldq, int orderQ)
{
    if (m < 0 || n < 0 || k < 0) return -1;
    if (orderA != ORACLE_ROW_MAJOR && orderA != ORACLE_COL_MAJOR) return -1;
    if (orderB != ORACLE_ROW_MAJOR && orderB != ORACLE_COL_MAJOR) return -1;
    if (orderQ != ORACLE_ROW_MAJOR && orderQ != ORACLE_COL_MAJOR) return -1;
    if (lda < (orderA == ORACLE_ROW_MAJOR ? k : m)) return -1;
    if (ldb < (orderB == ORACLE_ROW_MAJOR ? n : k)) return -1;
    if (ldq < (orderQ == ORACLE_ROW_MAJOR ? n : m)) return -1;
    if (!(scale == scale) || scale - scale != 0.0f) return -1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            uint32_t s = 0u;
            for (int64_t p = 0; p < k; ++p)
                s += widen(A, at(i, p, lda, orderA), a_unsigned)
                   * widen(B, at(p, j, ldb, orderB), b_unsigned);
            volatile float f = (float)(int32_t)s;   /* one rounding: int32 -> float32 */
            volatile float r = f * scale;           /* one rounding: float32 product   */
            float q = rintf(r);                     /* to an integer, ties to even     */
            if (q > 127.0f) q = 127.0f;
            if (q < -128.0f) q = -128.0f;
            Q[at(i, j, ldq, orderQ)] = (int8_t)q;
        }
    }
    return 0;
}

/* number of threads the parallel loop above runs with (for the bench report) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

/*
 * The same product with 16-bit operands, C (+)= A B with A and B of int16 and C of int32:
 * the (i32, i16, i16) forms of the paper's table of matrix-oriented instructions
 * (vpdpwssd, smopa).  Each int16 is widened to 32 bits before the multiply; products reach
 * 2^30, so sums wrap modulo 2^32 much sooner than with bytes (same reading as above).
 * lda, ldb count elements.
 */
int oracle_mip_gemm_s16(int64_t m, int64_t n, int64_t k,
                        const int16_t *A, int64_t lda, int orderA,
                        const int16_t *B, int64_t ldb, int orderB,
                        int32_t *C, int64_t ldc, int orderC,
                        int mode)
{
    if (m < 0 || n < 0 || k < 0) return -1;
    if (orderA != ORACLE_ROW_MAJOR && orderA != ORACLE_COL_MAJOR) return -1;
    if (orderB != ORACLE_ROW_MAJOR && orderB != ORACLE_COL_MAJOR) return -1;
    if (orderC != ORACLE_ROW_MAJOR && orderC != ORACLE_COL_MAJOR) return -1;
    if (mode != ORACLE_OVERWRITE && mode != ORACLE_ACCUMULATE) return -1;
    if (lda < (orderA == ORACLE_ROW_MAJOR ? k : m)) return -1;
    if (ldb < (orderB == ORACLE_ROW_MAJOR ? n : k)) return -1;
    if (ldc < (orderC == ORACLE_ROW_MAJOR ? n : m)) return -1;

    uint32_t *Cu = (uint32_t *)C;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        if (mode == ORACLE_OVERWRITE)
            for (int64_t j = 0; j < n; ++j)
                Cu[at(i, j, ldc, orderC)] = 0u;
        for (int64_t p = 0; p < k; ++p) {
            uint32_t a = (uint32_t)(int32_t)A[at(i, p, lda, orderA)];
            for (int64_t j = 0; j < n; ++j) {
                uint32_t b = (uint32_t)(int32_t)B[at(p, j, ldb, orderB)];
                Cu[at(i, j, ldc, orderC)] += a * b;
            }
        }
    }
    return 0;
}
