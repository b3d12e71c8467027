// Hardware characterisation: the rate of v_mfma_i32_32x32x32_i8 with every
// operand already in registers (no LDS, no memory traffic), on a 128 x 128
// accumulator block per wave, one wave per SIMD: the ceiling any GEMM kernel
// built on this instruction can approach on this device.  The rate depends
// strongly on the operand bits: the chip is power-limited, and random bytes
// toggle far more logic than near-zero ones.
#include "../../include/mipgemm.h"
#include "mip_internal.h"

namespace mip {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// pattern 0: operand registers hold small constants (mostly zero bits)
// pattern 1: operand registers hold random bytes that change every iteration,
//            as the fragments of a real k loop do
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iterations, int pattern, int *sink) {
  v16i acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0;
  v4i a[2][4], b[2][4];
  const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 977u;
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        a[s][f][r] = pattern ? (int)mix(seed + s * 64 + f * 8 + r) : r;
        b[s][f][r] = pattern ? (int)mix(seed + s * 64 + f * 8 + r + 4) : r + 4;
      }
  for (int it = 0; it < iterations; ++it) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int q = 0; q < 16; ++q)
        acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[s][q & 3], a[s][q >> 2], acc[q], 0, 0, 0);
    if (pattern) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          a[s][f] = a[s][f].yzwx;
          b[s][f] = b[s][f].wxyz;
        }
    }
  }
  int sum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) sum += acc[i][j];
  if (sum == 0x7fffffff) *sink = sum;  // keeps the accumulators live
}

}  // namespace mip

extern "C" int mipgemm_mfma_ceiling(int pattern, int iterations, void *stream, double *tops) {
  if (pattern != 0 && pattern != 1) return -1;
  if (iterations < 1 || iterations > 1000000) return -2;
  if (!tops) return -4;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int device = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&device);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
  if (e != hipSuccess) return (int)e;
  const int cus = prop.multiProcessorCount;
  int *sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  e = hipMalloc(&sink, sizeof(int));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  if (e == hipSuccess) {
    hipLaunchKernelGGL(mip::mfma_rate_kernel, dim3(cus), dim3(256), 0, s, iterations / 10 + 1,
                       pattern, sink);  // warm-up, also lets the clocks settle
    e = hipEventRecord(e0, s);
    hipLaunchKernelGGL(mip::mfma_rate_kernel, dim3(cus), dim3(256), 0, s, iterations, pattern, sink);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (e != hipSuccess) return (int)e;
  // one wave per SIMD, 4 SIMDs per compute unit, 2 * 128 * 128 * 64 operations per wave and iteration
  *tops = (double)cus * 4.0 * iterations * 2.0 * 128 * 128 * 64 / (ms * 1e-3) / 1e12;
  return 0;
}
