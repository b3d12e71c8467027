// Layout-agnostic kernels: the zero fill for k == 0 and a one-thread-per-element
// GEMM that accepts any strides and alignments.  The latter is the path of last
// resort and the in-library cross-check for the MFMA kernels; it is slow.
#include "mip_internal.h"

namespace mip {

__global__ __launch_bounds__(256) void fill_zero_kernel(int32_t *__restrict__ C, int64_t ldc,
                                                       int64_t m, int64_t n, int64_t c_sb) {
  C += (int64_t)blockIdx.z * c_sb;
  int64_t j = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
  int64_t i = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
  if (i < m && j < n) C[i * ldc + j] = 0;
}

// C(i,j) (+)= sum_p A(i,p) * B(p,j): the definition of the MIP GEMM (paper
// Section 5: INT8 products accumulated in INT32), one output element per thread.
__global__ __launch_bounds__(256) void simple_kernel(Problem p) {
  const int64_t j = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
  const int64_t i = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
  if (i >= p.m || j >= p.n) return;
  const int64_t z = blockIdx.z;  // problem of the batch
  const uint8_t *a = static_cast<const uint8_t *>(p.A) + z * p.a_sb + i * p.a_sm;
  const uint8_t *b = static_cast<const uint8_t *>(p.B) + z * p.b_sb + j * p.b_sn;
  uint32_t acc = 0;
  for (int64_t q = 0; q < p.k; ++q) {
    uint32_t av = a[q * p.a_sk], bv = b[q * p.b_sk];
    if (!p.a_unsigned) av = (uint32_t)(int32_t)(int8_t)av;
    if (!p.b_unsigned) bv = (uint32_t)(int32_t)(int8_t)bv;
    acc += av * bv;
  }
  if (p.out_float == 2) {  // requantised int8 output: clip(rint(float(sum) * scale))
    float r = __builtin_rintf(__fmul_rn((float)(int32_t)acc, p.scale));
    r = fminf(fmaxf(r, -128.0f), 127.0f);
    reinterpret_cast<int8_t *>(p.C)[z * p.c_sb + i * p.ldc + j] = (int8_t)(int)r;
    return;
  }
  uint32_t *c = reinterpret_cast<uint32_t *>(p.C) + z * p.c_sb + i * p.ldc + j;
  if (!p.out_float) {
    *c = p.accumulate ? *c + acc : acc;
  } else {  // dequantised output (paper Section 7.3): float(sum) * scale
    const float s = (float)(int32_t)acc;
    const float r = p.accumulate ? __fmaf_rn(s, p.scale, __uint_as_float(*c)) : __fmul_rn(s, p.scale);
    *c = __float_as_uint(r);
  }
}

// 64 columns x 4 rows per block; the caller keeps rows <= 65535 * 4
static dim3 grid_for(int64_t rows, int64_t n, int64_t batch) {
  return dim3((unsigned)((n + 63) / 64), (unsigned)((rows + 3) / 4), (unsigned)batch);
}

hipError_t launch_fill_zero(const Problem &p, hipStream_t s) {
  // rows go to grid.y, which holds 65535 blocks of 4 rows: cover taller
  // matrices in slabs
  const int64_t slab = 65535LL * 4;
  for (int64_t i0 = 0; i0 < p.m; i0 += slab) {
    int64_t rows = p.m - i0 < slab ? p.m - i0 : slab;
    dim3 grid = grid_for(rows, p.n, p.batch);
    hipLaunchKernelGGL(fill_zero_kernel, grid, dim3(256), 0, s, p.C + i0 * p.ldc, p.ldc, rows,
                       p.n, p.c_sb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_simple(const Problem &p, hipStream_t s) {
  const int64_t slab = 65535LL * 4;
  for (int64_t i0 = 0; i0 < p.m; i0 += slab) {
    Problem q = p;
    q.m = p.m - i0 < slab ? p.m - i0 : slab;
    q.A = static_cast<const uint8_t *>(p.A) + i0 * p.a_sm;
    q.C = p.out_float == 2 ? reinterpret_cast<int32_t *>(reinterpret_cast<int8_t *>(p.C) + i0 * p.ldc)
                           : p.C + i0 * p.ldc;
    dim3 grid = grid_for(q.m, q.n, q.batch);
    hipLaunchKernelGGL(simple_kernel, grid, dim3(256), 0, s, q);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace mip
