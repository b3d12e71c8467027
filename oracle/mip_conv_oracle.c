/*
 * CPU oracle for the steps around the MIP GEMM: the convolution lowering that
 * feeds it and the pre-packing of a weight matrix (end of the file).
 *
 * TEST INFRASTRUCTURE ONLY: the checker the GPU library is compared against;
 * the product never calls it, links it or falls back to it, and it shares no
 * code, header, table or helper with the HIP path.
 *
 * What it computes (paper, Section 7.2, the ResNet50 item: O = CONV(F, I) with
 * I of b images of h_i x w_i x c_i, F of c_o kernels of h_f x w_f x c_i, O of
 * b outputs of h_o x w_o x c_o; the lowering turns I into an augmented matrix
 * by IM2COL and the convolution into a GEMM of dimensions
 * (m, n, k) = (c_o, b h_o w_o, c_i h_f w_f)):
 *
 *   oracle_conv_direct: the convolution itself, as its definition, seven loops:
 *       O(g, oy, ox, o) [+]= sum_{y, x, c} F(o, y, x, c) * I(g, oy*s + y - p, ox*s + x - p, c)
 *     with positions outside the image contributing nothing.  F int8, I uint8
 *     (activations at face value, scale-only quantization of Section 7.3),
 *     sums in 32 bits wrapping modulo 2^32 as in the GEMM oracle.
 *
 *   oracle_im2col_u8: the augmented matrix, one row per output position
 *       M(n, kk) = I(g, oy*s + y - p, ox*s + x - p, c)   or 0 outside the image,
 *       n = (g*h_o + oy)*w_o + ox,    kk = (y*w_f + x)*c_i + c.
 *     Stored with kk contiguous and row pitch ldm: as the GEMM's B (k x n) that
 *     is column-major with ldb = ldm.
 *
 * The two functions share no loop: the lowering identity
 *   conv_direct(F, I) == GEMM(F as c_o x k row-major, im2col(I))
 * is one of the pins, next to hand-worked values, closed forms (delta and
 * all-ones filters, 1 x 1 filters, padding counts), stride subsampling and a
 * numpy sliding-window product (tests/test_conv_oracle_pins.py).
 *
 * Readings where the paper is silent:
 *   - tensors are stored with the index order the paper uses for their sizes,
 *     innermost last: I[g][iy][ix][c], F[o][y][x][c], O[g][oy][ox][o];
 *   - the k index of the lowered GEMM runs over (y, x, c) with c fastest, the n
 *     index over (g, oy, ox) with ox fastest;
 *   - one stride s >= 1 and one symmetric zero padding p >= 0 for both spatial
 *     dimensions, no dilation; h_o = floor((h_i + 2p - h_f) / s) + 1, same for w;
 *   - the padding value is the integer 0 (no zero point, Section 7.3);
 *   - the filter is applied without flipping it (the deep-learning convention:
 *     tap (y, x) meets the pixel y rows below and x columns right of the window's
 *     top-left corner).
 */
#include <stddef.h>
#include <stdint.h>

enum { CONV_OVERWRITE = 0, CONV_ACCUMULATE = 1 };

/* output extent along one dimension, or -1 when the filter does not fit */
static int64_t out_extent(int64_t in, int64_t f, int64_t s, int64_t p)
{
    int64_t span = in + 2 * p - f;
    if (span < 0) return -1;
    return span / s + 1;
}

int64_t oracle_conv_out_extent(int64_t in, int64_t f, int64_t s, int64_t p)
{
    if (in < 1 || f < 1 || s < 1 || p < 0) return -1;
    return out_extent(in, f, s, p);
}

static int bad_geometry(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                        int64_t hf, int64_t wf, int64_t s, int64_t p)
{
    if (b < 0 || hi < 1 || wi < 1 || ci < 1 || hf < 1 || wf < 1 || s < 1 || p < 0) return 1;
    if (out_extent(hi, hf, s, p) < 1 || out_extent(wi, wf, s, p) < 1) return 1;
    return 0;
}

int oracle_conv_direct(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                       int64_t co, int64_t hf, int64_t wf, int64_t s, int64_t p,
                       const int8_t *F, const uint8_t *I, int32_t *O, int mode)
{
    if (bad_geometry(b, hi, wi, ci, hf, wf, s, p) || co < 0) return -1;
    if (mode != CONV_OVERWRITE && mode != CONV_ACCUMULATE) return -1;
    const int64_t ho = out_extent(hi, hf, s, p), wo = out_extent(wi, wf, s, p);
    uint32_t *Ou = (uint32_t *)O;

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t g = 0; g < b; ++g)
        for (int64_t oy = 0; oy < ho; ++oy)
            for (int64_t ox = 0; ox < wo; ++ox)
                for (int64_t o = 0; o < co; ++o) {
                    uint32_t sum = 0u;
                    for (int64_t y = 0; y < hf; ++y) {
                        const int64_t iy = oy * s + y - p;
                        if (iy < 0 || iy >= hi) continue;
                        for (int64_t x = 0; x < wf; ++x) {
                            const int64_t ix = ox * s + x - p;
                            if (ix < 0 || ix >= wi) continue;
                            for (int64_t c = 0; c < ci; ++c) {
                                uint32_t f = (uint32_t)(int32_t)F[((o * hf + y) * wf + x) * ci + c];
                                uint32_t v = (uint32_t)I[((g * hi + iy) * wi + ix) * ci + c];
                                sum += f * v;
                            }
                        }
                    }
                    const size_t at = (size_t)(((g * ho + oy) * wo + ox) * co + o);
                    if (mode == CONV_ACCUMULATE) Ou[at] += sum;
                    else Ou[at] = sum;
                }
    return 0;
}

int oracle_im2col_u8(int64_t b, int64_t hi, int64_t wi, int64_t ci,
                     int64_t hf, int64_t wf, int64_t s, int64_t p,
                     const uint8_t *I, uint8_t *M, int64_t ldm)
{
    if (bad_geometry(b, hi, wi, ci, hf, wf, s, p)) return -1;
    const int64_t ho = out_extent(hi, hf, s, p), wo = out_extent(wi, wf, s, p);
    const int64_t k = hf * wf * ci;
    if (ldm < k) return -1;

    for (int64_t g = 0; g < b; ++g)
        for (int64_t oy = 0; oy < ho; ++oy)
            for (int64_t ox = 0; ox < wo; ++ox) {
                uint8_t *row = M + (size_t)(((g * ho + oy) * wo + ox) * ldm);
                for (int64_t y = 0; y < hf; ++y)
                    for (int64_t x = 0; x < wf; ++x)
                        for (int64_t c = 0; c < ci; ++c) {
                            const int64_t iy = oy * s + y - p, ix = ox * s + x - p;
                            uint8_t v = 0;
                            if (iy >= 0 && iy < hi && ix >= 0 && ix < wi)
                                v = I[((g * hi + iy) * wi + ix) * ci + c];
                            row[(y * wf + x) * ci + c] = v;
                        }
            }
    return 0;
}

/*
 * Weight pre-packing: the k x n 8-bit matrix B, stored in either order, rewritten
 * with k contiguous (column-major, pitch ldp >= k) -- the form in which the paper's
 * packed buffer B_c feeds the micro-kernel (Section 4.1: packing makes the
 * micro-kernel's accesses unit-stride, its cost amortised over the reuse of B_c;
 * Section 5 notes that every MIP instruction wants k contiguous per operand
 * register).  Pure data movement: P(p, j) = B(p, j).  Bytes of P beyond the k
 * entries of a column are not written.  order: 0 row-major B(p,j) = B[p*ldb + j],
 * 1 column-major B(p,j) = B[p + j*ldb].
 */
int oracle_pack_b(int64_t k, int64_t n, const uint8_t *B, int64_t ldb, int order,
                  uint8_t *P, int64_t ldp)
{
    if (k < 0 || n < 0 || (order != 0 && order != 1)) return -1;
    if (ldb < (order == 0 ? n : k) || ldp < k) return -1;
    for (int64_t j = 0; j < n; ++j)
        for (int64_t p = 0; p < k; ++p)
            P[(size_t)(j * ldp + p)] = order == 0 ? B[(size_t)(p * ldb + j)]
                                                  : B[(size_t)(p + j * ldb)];
    return 0;
}

/*
 * The k-sums of a signed 8-bit weight matrix: s(j) = sum over p of B(p, j), one per column,
 * kept with the packed weights (Section 4.1's packed buffer carried to constant weights: what
 * depends on B alone is computed once).  With activations that are unsigned bytes the integer
 * product can be formed from the activations moved into the signed range,
 *     sum_p a(p) b(p, j) = sum_p (a(p) - 128) b(p, j) + 128 s(j),
 * which is the identity the pins check against the GEMM oracle.  The sums are kept in 32
 * bits and wrap modulo 2^32 like every other sum here.  order as in oracle_pack_b.
 */
int oracle_column_sums_s8(int64_t k, int64_t n, const int8_t *B, int64_t ldb, int order,
                          int32_t *s)
{
    if (k < 0 || n < 0 || (order != 0 && order != 1)) return -1;
    if (ldb < (order == 0 ? n : k)) return -1;
    for (int64_t j = 0; j < n; ++j) {
        uint32_t sum = 0;
        for (int64_t p = 0; p < k; ++p) {
            const int8_t b = order == 0 ? B[(size_t)(p * ldb + j)] : B[(size_t)(p + j * ldb)];
            sum += (uint32_t)(int32_t)b;
        }
        s[j] = (int32_t)sum;
    }
    return 0;
}
