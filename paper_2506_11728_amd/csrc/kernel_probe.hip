// Hardware characterisation: the rate of v_mfma_i32_32x32x32_i8 and of
// v_mfma_i32_16x16x64_i8 with every operand already in registers (no LDS, no
// memory traffic), on a 128 x 128 accumulator block per wave, one wave per SIMD:
// the ceiling any GEMM kernel built on these instructions can approach on this
// device.  The rate depends
// strongly on the operand bits: the chip is power-limited, and random bytes
// toggle far more logic than near-zero ones.  Every workgroup also reads the
// shader clock counter and the constant 100 MHz counter around its loop, so the
// clock the device actually ran at comes back with the rate.
#include "../../include/mipgemm.h"
#include "mip_internal.h"

namespace mip {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// PATTERN 0: operand registers hold small constants (mostly zero bits).
// PATTERN 1: random bytes, rotated inside each operand between iterations: the operands
//            change as the fragments of a k loop do, but 128 register moves are issued
//            between the 32 matrix instructions of an iteration.
// PATTERN 2: random bytes, SETS = 2 fixed operand sets used in turn: nothing but matrix
//            instructions in the loop.
// PATTERN 3: random bytes, SETS = 6 fixed operand sets used in turn (192 operand
//            registers beside the 256 accumulators): as 2, with three times as many
//            distinct operand values passing through the matrix pipe.
// PATTERN 4: as 0, PATTERN 5: as 2 with one operand set, on v_mfma_i32_16x16x64_i8 (64
//            four-register accumulators, 8 + 8 operand fragments): the same multiply-
//            accumulates per clock on paper, but a quarter of the accumulator registers
//            read and written per multiply-accumulate.
// One iteration is always 128 x 128 x 64 multiply-accumulates (32 or 64 matrix instructions).
template <int PATTERN>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iterations, int *sink,
                                                        unsigned long long *clocks) {
  constexpr int SETS = PATTERN == 3 ? 6 : 2;
  v16i acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0;
  v4i a[SETS][4], b[SETS][4];
  const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 977u;
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        a[s][f][r] = PATTERN ? (int)mix(seed + s * 64 + f * 8 + r) : r;
        b[s][f][r] = PATTERN ? (int)mix(seed + s * 64 + f * 8 + r + 4) : r + 4;
      }
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
  // SETS / 2 iterations per trip, so that every trip walks through all the sets
  for (int it = 0; it < iterations; it += SETS / 2) {
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
      for (int q = 0; q < 16; ++q)
        acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[s][q & 3], a[s][q >> 2], acc[q], 0, 0, 0);
    if (PATTERN == 1) {
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
  if (clocks && threadIdx.x == 0) {
    clocks[2 * blockIdx.x] = __builtin_readcyclecounter() - c0;
    clocks[2 * blockIdx.x + 1] = wall_clock64() - r0;
  }
}

template <int RANDOM>
__global__ __launch_bounds__(256) void mfma16_rate_kernel(int iterations, int *sink,
                                                          unsigned long long *clocks) {
  v4i acc[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) acc[i] = v4i{0, 0, 0, 0};
  v4i a[8], b[8];
  const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 977u;
#pragma unroll
  for (int f = 0; f < 8; ++f)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      a[f][r] = RANDOM ? (int)mix(seed + f * 8 + r) : r;
      b[f][r] = RANDOM ? (int)mix(seed + f * 8 + r + 4) : r + 4;
    }
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
  for (int it = 0; it < iterations; ++it) {
#pragma unroll
    for (int q = 0; q < 64; ++q)
      acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b[q & 7], a[q >> 3], acc[q], 0, 0, 0);
  }
  int sum = 0;
#pragma unroll
  for (int i = 0; i < 64; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) sum += acc[i][j];
  if (sum == 0x7fffffff) *sink = sum;  // keeps the accumulators live
  if (clocks && threadIdx.x == 0) {
    clocks[2 * blockIdx.x] = __builtin_readcyclecounter() - c0;
    clocks[2 * blockIdx.x + 1] = wall_clock64() - r0;
  }
}

}  // namespace mip

extern "C" int mipgemm_mfma_ceiling_clocked(int pattern, int iterations, void *stream,
                                            double *tops, double *shader_mhz) {
  if (pattern < 0 || pattern > 5) return -1;
  if (iterations < 1 || iterations > 1000000) return -2;
  if (!tops) return -4;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int device = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&device);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
  if (e != hipSuccess) return (int)e;
  const int cus = prop.multiProcessorCount;
  iterations = (iterations + 2) / 3 * 3;  // whole trips for every pattern
  void (*kern)(int, int *, unsigned long long *) =
      pattern == 0 ? mip::mfma_rate_kernel<0>
                   : (pattern == 1 ? mip::mfma_rate_kernel<1>
                                   : (pattern == 2 ? mip::mfma_rate_kernel<2> : mip::mfma_rate_kernel<3>));
  if (pattern == 4) kern = mip::mfma16_rate_kernel<0>;
  if (pattern == 5) kern = mip::mfma16_rate_kernel<1>;
  int *sink = nullptr;
  unsigned long long *clocks = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  e = hipMalloc(&sink, sizeof(int));
  if (e == hipSuccess) e = hipMalloc(&clocks, sizeof(unsigned long long) * 2 * cus);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  double cycles = 0.0, ticks = 0.0;
  if (e == hipSuccess) {
    // warm-up: a tenth of the work, which also lets the clocks settle
    hipLaunchKernelGGL(kern, dim3(cus), dim3(256), 0, s, (iterations / 30 + 1) * 3, sink, clocks);
    e = hipEventRecord(e0, s);
    hipLaunchKernelGGL(kern, dim3(cus), dim3(256), 0, s, iterations, sink, clocks);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess && shader_mhz) {
      unsigned long long *host =
          static_cast<unsigned long long *>(malloc(sizeof(unsigned long long) * 2 * cus));
      if (host) {
        e = hipMemcpy(host, clocks, sizeof(unsigned long long) * 2 * cus, hipMemcpyDeviceToHost);
        for (int i = 0; e == hipSuccess && i < cus; ++i) {
          cycles += (double)host[2 * i];
          ticks += (double)host[2 * i + 1];
        }
        free(host);
      }
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (clocks) (void)hipFree(clocks);
  if (e != hipSuccess) return (int)e;
  // one wave per SIMD, 4 SIMDs per compute unit, 2 * 128 * 128 * 64 operations per wave and iteration
  *tops = (double)cus * 4.0 * iterations * 2.0 * 128 * 128 * 64 / (ms * 1e-3) / 1e12;
  if (shader_mhz) *shader_mhz = ticks > 0.0 ? cycles / ticks * 100.0 : 0.0;  // ticks of 10 ns
  return 0;
}

extern "C" int mipgemm_mfma_ceiling(int pattern, int iterations, void *stream, double *tops) {
  if (pattern != 0 && pattern != 1) return -1;
  return mipgemm_mfma_ceiling_clocked(pattern, iterations, stream, tops, nullptr);
}
