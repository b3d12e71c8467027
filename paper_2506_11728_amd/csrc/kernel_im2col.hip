// The lowering step of a convolution written out (paper Section 7.2: the input tensor
// becomes an augmented matrix through IM2COL and the convolution a GEMM with
// (m, n, k) = (c_o, b h_o w_o, c_i h_f w_f)): row n = (g, oy, ox) of M holds, for
// k = (y, x, c) with c fastest, pixel (g, oy*stride + y - pad, ox*stride + x - pad, c)
// of the image tensor, or 0 where the tap falls outside the image.
//
// Pure data movement, bound by the write of M (h_f w_f times the size of the
// image).  Each thread moves UNIT bytes: 16 when the channel count, the row pitch
// and both bases allow aligned 16-byte accesses, else 1.  A workgroup covers whole
// rows of M, so that the division of a row index into (g, oy, ox) happens once
// per row and thread, not once per byte.
#include "mip_internal.h"

namespace mip {

namespace {

typedef int v4i_copy __attribute__((ext_vector_type(4)));

template <int UNIT>
__global__ __launch_bounds__(256) void im2col_kernel(ConvGeom G, int64_t rows, int units_per_row,
                                                     const uint8_t *I, uint8_t *M, int64_t ldm) {
  // threads_per_row threads share a row; a workgroup takes 256 / threads_per_row rows at a time
  const int threads_per_row = units_per_row < 256 ? units_per_row : 256;
  const int rows_per_pass = 256 / threads_per_row;
  const int r_local = threadIdx.x / threads_per_row;
  const int u_first = threadIdx.x - r_local * threads_per_row;
  if (r_local >= rows_per_pass) return;
  const int per_image = G.ho * G.wo;
  for (int64_t row = (int64_t)blockIdx.x * rows_per_pass + r_local; row < rows;
       row += (int64_t)gridDim.x * rows_per_pass) {
    const int g = (int)row / per_image;  // the host keeps the row count below 2^31
    const int r = (int)row - g * per_image;
    const int oy = r / G.wo, ox = r - oy * G.wo;
    const int iy0 = oy * G.stride - G.pad, ix0 = ox * G.stride - G.pad;
    const uint8_t *image = I + (int64_t)g * G.hi * G.wi * G.ci;
    uint8_t *out = M + row * ldm;
    for (int u = u_first; u < units_per_row; u += threads_per_row) {
      const int kk = u * UNIT;
      const int tap = kk / G.ci, c = kk - tap * G.ci;
      const int y = tap / G.wf, x = tap - y * G.wf;
      const int iy = iy0 + y, ix = ix0 + x;
      const bool inside = (unsigned)iy < (unsigned)G.hi && (unsigned)ix < (unsigned)G.wi;
      const uint8_t *src = image + ((int64_t)iy * G.wi + ix) * G.ci + c;
      if (UNIT == 16) {
        v4i_copy v = {0, 0, 0, 0};
        if (inside) v = *reinterpret_cast<const v4i_copy *>(src);
        __builtin_nontemporal_store(v, reinterpret_cast<v4i_copy *>(out + kk));
      } else {
        out[kk] = inside ? *src : (uint8_t)0;
      }
    }
  }
}

}  // namespace

hipError_t launch_im2col(const ConvGeom &g, int64_t rows, int64_t k, const uint8_t *I, uint8_t *M,
                         int64_t ldm, hipStream_t s) {
  if (rows == 0 || k == 0) return hipSuccess;
  const bool wide = g.ci % 16 == 0 && ldm % 16 == 0 && reinterpret_cast<uintptr_t>(I) % 16 == 0 &&
                    reinterpret_cast<uintptr_t>(M) % 16 == 0;
  const int64_t units = wide ? k / 16 : k;
  const int threads_per_row = units < 256 ? (int)units : 256;
  const int rows_per_pass = 256 / threads_per_row;
  int64_t blocks = (rows + rows_per_pass - 1) / rows_per_pass;
  if (blocks > 256 * 64) blocks = 256 * 64;  // the row loop strides over the rest
  if (wide)
    hipLaunchKernelGGL(im2col_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, s, g, rows,
                       (int)units, I, M, ldm);
  else
    hipLaunchKernelGGL(im2col_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, s, g, rows,
                       (int)units, I, M, ldm);
  return hipGetLastError();
}

}  // namespace mip
