// 16-bit operands on the 8-bit matrix instructions: byte planes.
//
// gfx950 has no integer matrix instruction for 16-bit operands (the paper's ISA table lists
// (i32, i16, i16) forms for other machines: vpdpwssd, smopa), so an int16 x int16 -> int32
// product is built from int8 products.  With x' = x - 128, every int16 splits exactly into two
// SIGNED bytes, x' = 256 h + l with h = x >> 8 (arithmetic) and l = (x & 255) - 128, and
//     sum_p a b = sum_p a' b' + 128 (sum_p a' + sum_p b') + 16384 k,
//     sum_p a' b' = 65536 sum_p ah bh + 256 sum_p (ah bl + al bh) + sum_p al bl,
// all modulo 2^32.  The three byte products are ordinary s8 x s8 GEMMs on the planes (the
// middle one with the planes side by side along k), run by the kernels of the 8-bit path; the
// kernels here only split the operands into planes and put the pieces together.
#include "mip_internal.h"

namespace mip {

namespace {

struct __attribute__((packed, aligned(2))) s16x8 { short v[8]; };
typedef int v4i_s16 __attribute__((ext_vector_type(4)));

// Operand X (rows x k, element (r, p) at X[r * s_r + p * s_k], one of the strides 1) into the
// plane matrix P: row r holds kp bytes of the first plane, then kp bytes of the second, zeros
// from p = k on.  hi_first: the high bytes come first (A), else the low bytes (B), so that
// [A planes] . [B planes] along 2 kp is sum ah bl + al bh.  One thread per 16 consecutive p
// of one row; with a strided operand consecutive threads take consecutive rows.
__global__ __launch_bounds__(256) void split_planes_kernel(const int16_t *X, int64_t s_r, int64_t s_k,
                                                           int64_t rows, int64_t k, int64_t kp,
                                                           uint8_t *P, int hi_first) {
  const int64_t chunks = kp / 16;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t r, c;
  if (s_k == 1) { r = t / chunks; c = t % chunks; } else { c = t / rows; r = t % rows; }
  if (r >= rows || c >= chunks) return;
  const int64_t p0 = c * 16;
  union { v4i_s16 v; uint8_t b[16]; } hi, lo;
  hi.v = v4i_s16{0, 0, 0, 0};
  lo.v = v4i_s16{0, 0, 0, 0};
  if (s_k == 1 && p0 + 16 <= k) {
    const s16x8 x0 = *reinterpret_cast<const s16x8 *>(X + r * s_r + p0);
    const s16x8 x1 = *reinterpret_cast<const s16x8 *>(X + r * s_r + p0 + 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      hi.b[e] = (uint8_t)(x0.v[e] >> 8);
      lo.b[e] = (uint8_t)((x0.v[e] & 255) ^ 128);
      hi.b[8 + e] = (uint8_t)(x1.v[e] >> 8);
      lo.b[8 + e] = (uint8_t)((x1.v[e] & 255) ^ 128);
    }
  } else {
    for (int e = 0; e < 16; ++e) {
      if (p0 + e < k) {
        const int x = X[r * s_r + (p0 + e) * s_k];
        hi.b[e] = (uint8_t)(x >> 8);
        lo.b[e] = (uint8_t)((x & 255) ^ 128);
      }
    }
  }
  uint8_t *row = P + r * (2 * kp) + p0;
  *reinterpret_cast<v4i_s16 *>(row + (hi_first ? 0 : kp)) = hi.v;
  *reinterpret_cast<v4i_s16 *>(row + (hi_first ? kp : 0)) = lo.v;
}

// C(i, j) = [C(i, j) +] 65536 T1 + 256 T2 + T3 + 128 (256 sAh(i) + sAl(i) + 256 sBh(j) + sBl(j))
// + 16384 k, modulo 2^32; the T are m x n, row-major, dense.  The plane sums come as the byte
// sums of the plane matrices taken as columns of kp bytes: sA[2 i] = sAh(i), sA[2 i + 1] =
// sAl(i); sB[2 j] = sBl(j), sB[2 j + 1] = sBh(j).  Four columns per thread; WIDE: n and ldc
// multiples of 4 and C 16-byte aligned, so that every access is one 16-byte piece.
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

template <bool WIDE>
__global__ __launch_bounds__(256) void combine_planes_kernel(const uint32_t *T1, const uint32_t *T2,
                                                             const uint32_t *T3, const int32_t *sA,
                                                             const int32_t *sB, int64_t m, int64_t n,
                                                             uint32_t k, uint32_t *C, int64_t ldc,
                                                             int accumulate) {
  const int64_t quads = (n + 3) / 4;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i = t / quads, j0 = (t % quads) * 4;
  if (i >= m) return;
  const uint32_t row = 128u * (256u * (uint32_t)sA[2 * i] + (uint32_t)sA[2 * i + 1]) + 16384u * k;
  const int64_t at = i * n + j0;
  if (WIDE) {
    const v4u t1 = *reinterpret_cast<const v4u *>(T1 + at), t2 = *reinterpret_cast<const v4u *>(T2 + at),
              t3 = *reinterpret_cast<const v4u *>(T3 + at);
    const v4u b0 = *reinterpret_cast<const v4u *>(sB + 2 * j0), b1 = *reinterpret_cast<const v4u *>(sB + 2 * j0 + 4);
    const v4u col = {128u * (256u * b0[1] + b0[0]), 128u * (256u * b0[3] + b0[2]),
                     128u * (256u * b1[1] + b1[0]), 128u * (256u * b1[3] + b1[2])};
    v4u v = (t1 << 16) + (t2 << 8) + t3 + col + row;
    v4u *c = reinterpret_cast<v4u *>(C + i * ldc + j0);
    if (accumulate) v += *c;
    *c = v;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t j = j0 + e;
      if (j >= n) break;
      uint32_t v = (T1[at + e] << 16) + (T2[at + e] << 8) + T3[at + e] + row +
                   128u * (256u * (uint32_t)sB[2 * j + 1] + (uint32_t)sB[2 * j]);
      if (accumulate) v += C[i * ldc + j];
      C[i * ldc + j] = v;
    }
  }
}

}  // namespace

hipError_t launch_split_planes(const int16_t *X, int64_t s_r, int64_t s_k, int64_t rows, int64_t k,
                               int64_t kp, uint8_t *P, bool hi_first, hipStream_t s) {
  const int64_t threads = rows * (kp / 16);
  if (threads <= 0) return hipSuccess;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff || kp % 16) return hipErrorInvalidValue;
  hipLaunchKernelGGL(split_planes_kernel, dim3((unsigned)blocks), dim3(256), 0, s, X, s_r, s_k, rows, k, kp,
                     P, hi_first ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_combine_planes(const int32_t *T1, const int32_t *T2, const int32_t *T3,
                                 const int32_t *sA, const int32_t *sB, int64_t m, int64_t n, int64_t k,
                                 int32_t *C, int64_t ldc, bool accumulate, hipStream_t s) {
  const int64_t threads = m * ((n + 3) / 4);
  if (threads <= 0) return hipSuccess;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  auto aligned16 = [](const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  const bool wide = n % 4 == 0 && ldc % 4 == 0 && aligned16(C) && aligned16(T1) && aligned16(T2) &&
                    aligned16(T3) && aligned16(sB);
  auto kern = wide ? combine_planes_kernel<true> : combine_planes_kernel<false>;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, s,
                     reinterpret_cast<const uint32_t *>(T1), reinterpret_cast<const uint32_t *>(T2),
                     reinterpret_cast<const uint32_t *>(T3), sA, sB, m, n, (uint32_t)k,
                     reinterpret_cast<uint32_t *>(C), ldc, accumulate ? 1 : 0);
  return hipGetLastError();
}

}  // namespace mip
