// The lowering step of a convolution written out (paper Section 7.2: the input tensor
// becomes an augmented matrix through IM2COL and the convolution a GEMM with
// (m, n, k) = (c_o, b h_o w_o, c_i h_f w_f)): row n = (g, oy, ox) of M holds, for
// k = (y, x, c) with c fastest, pixel (g, oy*stride + y - pad, ox*stride + x - pad, c)
// of the image tensor, or 0 where the tap falls outside the image.
//
// Pure data movement, bound by the write of M (h_f w_f times the size of the
// image).  Each thread produces 16 consecutive bytes of a row of M at a time: one
// 16-byte load when they are 16 channels of one tap (channel count a multiple of
// 16, aligned image), else gathered byte by byte (the 3-channel first layer of a
// network); one 16-byte store when the row pitch and the base of M allow it.  A
// workgroup covers whole rows of M, four at a time per thread, so that the split
// of a row index into (g, oy, ox) and of a byte position into (y, x, c) happens
// once per 16 bytes or less, and four loads are in flight before the first store.
#include "mip_internal.h"

namespace mip {

namespace {

typedef int v4i_copy __attribute__((ext_vector_type(4)));

constexpr int ROWS_IN_FLIGHT = 4;  // rows a thread fetches before it stores any

union Piece {  // 16 bytes of a row of M
  v4i_copy v;
  uint8_t b[16];
};

// WIDE_LOAD: c_i % 16 == 0 and the image is 16-byte aligned.  WIDE_STORE: ldm % 16 == 0
// and M is 16-byte aligned.
// kfill >= k: bytes k .. kfill - 1 of every row are written as zeros (kfill == k: none).
template <bool WIDE_LOAD, bool WIDE_STORE>
__global__ __launch_bounds__(256) void im2col_kernel(ConvGeom G, int64_t rows, int k, int kfill,
                                                     const uint8_t *I, uint8_t *M, int64_t ldm) {
  // threads_per_row threads share a row; a workgroup takes 256 / threads_per_row rows at a
  // time, ROWS_IN_FLIGHT times over, each thread keeping its position inside the row
  const int pieces_per_row = (kfill + 15) / 16;
  const int threads_per_row = pieces_per_row < 256 ? pieces_per_row : 256;
  const int rows_per_pass = 256 / threads_per_row;
  const int r_local = threadIdx.x / threads_per_row;
  const int u_first = threadIdx.x - r_local * threads_per_row;
  if (r_local >= rows_per_pass) return;
  const int per_image = G.ho * G.wo;
  const int64_t rows_per_block = (int64_t)rows_per_pass * ROWS_IN_FLIGHT;
  for (int64_t row0 = (int64_t)blockIdx.x * rows_per_block + r_local; row0 < rows;
       row0 += (int64_t)gridDim.x * rows_per_block) {
    // where the window of each row starts (top-left tap; may lie outside the image)
    int iy0[ROWS_IN_FLIGHT], ix0[ROWS_IN_FLIGHT];
    int64_t image[ROWS_IN_FLIGHT];
#pragma unroll
    for (int j = 0; j < ROWS_IN_FLIGHT; ++j) {
      int64_t row = row0 + (int64_t)j * rows_per_pass;
      if (row >= rows) row = rows - 1;  // computed, not stored
      const int g = (int)row / per_image;  // the host keeps the row count below 2^31
      const int r = (int)row - g * per_image;
      const int oy = r / G.wo, ox = r - oy * G.wo;
      iy0[j] = oy * G.stride - G.pad;
      ix0[j] = ox * G.stride - G.pad;
      image[j] = (int64_t)g * G.hi * G.wi * G.ci;
    }
    for (int u = u_first; u < pieces_per_row; u += threads_per_row) {
      const int kk = u * 16;
      const int valid = k - kk < 16 ? k - kk : 16;  // bytes of this piece that belong to the row (may be <= 0)
      const int written = kfill - kk < 16 ? kfill - kk : 16;  // bytes of it that are stored
      const int tap = kk / G.ci, c = kk - tap * G.ci;
      const int y = tap / G.wf, x = tap - y * G.wf;
      Piece piece[ROWS_IN_FLIGHT];
#pragma unroll
      for (int j = 0; j < ROWS_IN_FLIGHT; ++j) {
        const uint8_t *base = I + image[j];
        if (WIDE_LOAD) {
          const int iy = iy0[j] + y, ix = ix0[j] + x;
          const bool inside = valid > 0 && (unsigned)iy < (unsigned)G.hi && (unsigned)ix < (unsigned)G.wi;
          piece[j].v = v4i_copy{0, 0, 0, 0};
          if (inside)
            piece[j].v = *reinterpret_cast<const v4i_copy *>(base + ((int64_t)iy * G.wi + ix) * G.ci + c);
        } else {
          int yy = y, xx = x, cc = c;  // walk (y, x, c) along the 16 bytes
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int iy = iy0[j] + yy, ix = ix0[j] + xx;
            const bool inside = e < valid && (unsigned)iy < (unsigned)G.hi &&
                                (unsigned)ix < (unsigned)G.wi;
            piece[j].b[e] = inside ? base[((int64_t)iy * G.wi + ix) * G.ci + cc] : (uint8_t)0;
            if (++cc == G.ci) {
              cc = 0;
              if (++xx == G.wf) {
                xx = 0;
                ++yy;
              }
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < ROWS_IN_FLIGHT; ++j) {
        const int64_t row = row0 + (int64_t)j * rows_per_pass;
        if (row < rows) {
          uint8_t *out = M + row * ldm + kk;
          if (WIDE_STORE && written == 16) {
            *reinterpret_cast<v4i_copy *>(out) = piece[j].v;
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e)
              if (e < written) out[e] = piece[j].b[e];
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_im2col(const ConvGeom &g, int64_t rows, int64_t k, const uint8_t *I, uint8_t *M,
                         int64_t ldm, hipStream_t s, int64_t kfill) {
  if (kfill < k) kfill = k;
  if (rows == 0 || k == 0) return hipSuccess;
  const bool wide_load = g.ci % 16 == 0 && reinterpret_cast<uintptr_t>(I) % 16 == 0;
  const bool wide_store = ldm % 16 == 0 && reinterpret_cast<uintptr_t>(M) % 16 == 0;
  const int64_t pieces = (kfill + 15) / 16;
  const int threads_per_row = pieces < 256 ? (int)pieces : 256;
  const int64_t rows_per_block = (int64_t)(256 / threads_per_row) * ROWS_IN_FLIGHT;
  int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
  if (blocks > 256 * 64) blocks = 256 * 64;  // the row loop strides over the rest
  void (*kern)(ConvGeom, int64_t, int, int, const uint8_t *, uint8_t *, int64_t) =
      wide_load ? (wide_store ? im2col_kernel<true, true> : im2col_kernel<true, false>)
                : (wide_store ? im2col_kernel<false, true> : im2col_kernel<false, false>);
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, s, g, rows, (int)k, (int)kfill, I, M, ldm);
  return hipGetLastError();
}

}  // namespace mip
