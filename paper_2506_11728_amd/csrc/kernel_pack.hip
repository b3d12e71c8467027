// Weight pre-packing: the k x n 8-bit matrix B rewritten once with k contiguous
// (column-major, pitch ldp), the form in which the paper's packed buffer B_c
// feeds its micro-kernels (Section 4.1; Section 5: every MIP instruction wants k
// contiguous per operand register).  The GEMM kernels take either order as it is,
// so this is never needed for correctness; it pays when the same weights meet a
// few rows of activations many times, because the skinny-m kernel streams a
// k-contiguous B in whole 64-byte runs and a row-major one in 16-byte pieces.
//
// Pure data movement: a byte transpose of 64 x 64 tiles through LDS (16-byte
// loads along n at whatever alignment, 16-byte stores along k where alignment
// allows, single bytes at ragged edges), or a re-pitching copy when B already
// is k-contiguous.  The same kernels pack both operands of a GEMM whose storage
// the direct-to-LDS kernels cannot stream (Section 4.1: Pack A, Pack B into the
// aligned buffers A_c, B_c): then the k tail up to the padded length is zeroed.
#include "mip_internal.h"

namespace mip {

namespace {

typedef int v4i_pack __attribute__((ext_vector_type(4)));
struct __attribute__((packed, aligned(1))) unaligned_piece { v4i_pack v; };
constexpr int PT = 64;      // tile edge
constexpr int PITCH = 80;   // LDS row pitch: a multiple of 16 that staggers the banks

// B(p, j) = B[p * ldb + j]  ->  P[j * ldp + p]
// Entries k .. kfill - 1 of every packed column are written as zeros (kfill == k: none).
__global__ __launch_bounds__(256) void pack_transpose_kernel(int64_t k, int64_t kfill, int64_t n,
                                                             const uint8_t *B, int64_t ldb,
                                                             uint8_t *P, int64_t ldp,
                                                             int wide_load, int wide_store,
                                                             int tiles_n) {
  __shared__ __attribute__((aligned(16))) uint8_t tile[PT * PITCH];
  const int t = threadIdx.x;
  const int64_t p0 = (int64_t)(blockIdx.x / tiles_n) * PT, n0 = (int64_t)(blockIdx.x % tiles_n) * PT;
  {
    const int p = t >> 2, c = (t & 3) * 16;  // k row of the tile, first of 16 columns
    const int64_t row = p0 + p, col = n0 + c;
    union { v4i_pack v; uint8_t b[16]; } piece;
    piece.v = v4i_pack{0, 0, 0, 0};
    if (row < k) {
      const uint8_t *src = B + row * ldb + col;
      if (col + 16 <= n) {
        if (wide_load) piece.v = *reinterpret_cast<const v4i_pack *>(src);
        else piece.v = reinterpret_cast<const unaligned_piece *>(src)->v;
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (col + e < n) piece.b[e] = src[e];
      }
    }
    *reinterpret_cast<v4i_pack *>(tile + p * PITCH + c) = piece.v;
  }
  __syncthreads();
  {
    const int j = t >> 2, q = (t & 3) * 16;  // column of the tile, first of 16 k rows
    const int64_t col = n0 + j, row = p0 + q;
    if (col < n && row < kfill) {
      union { v4i_pack v; uint8_t b[16]; } piece;  // rows at k and beyond were staged as zeros
#pragma unroll
      for (int e = 0; e < 16; ++e) piece.b[e] = tile[(q + e) * PITCH + j];
      uint8_t *dst = P + col * ldp + row;
      if (wide_store && row + 16 <= kfill) {
        *reinterpret_cast<v4i_pack *>(dst) = piece.v;
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (row + e < kfill) dst[e] = piece.b[e];
      }
    }
  }
}

// B already k-contiguous: column j moves from B + j * ldb to P + j * ldp
// wide_load / wide_store: the source / the destination is 16-byte aligned, pitch included
__global__ __launch_bounds__(256) void pack_copy_kernel(int64_t k, int64_t kfill, int64_t n,
                                                        const uint8_t *B, int64_t ldb, uint8_t *P,
                                                        int64_t ldp, int wide_load, int wide_store) {
  const int64_t pieces = (kfill + 15) / 16;
  const int64_t total = pieces * n;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t j = i / pieces, p = (i - j * pieces) * 16;
    const uint8_t *src = B + j * ldb + p;
    uint8_t *dst = P + j * ldp + p;
    union { v4i_pack v; uint8_t b[16]; } piece;
    piece.v = v4i_pack{0, 0, 0, 0};
    if (p + 16 <= k) {
      if (wide_load) piece.v = *reinterpret_cast<const v4i_pack *>(src);
      else piece.v = reinterpret_cast<const unaligned_piece *>(src)->v;
    } else {
      for (int e = 0; e < 16 && p + e < k; ++e) piece.b[e] = src[e];
    }
    if (wide_store && p + 16 <= kfill) {
      *reinterpret_cast<v4i_pack *>(dst) = piece.v;
    } else {
      for (int e = 0; e < 16 && p + e < kfill; ++e) dst[e] = piece.b[e];
    }
  }
}

bool aligned16(const void *p, int64_t ld) {
  return reinterpret_cast<uintptr_t>(p) % 16 == 0 && ld % 16 == 0;
}

}  // namespace

hipError_t launch_pack_b(int64_t k, int64_t n, const uint8_t *B, int64_t ldb, bool b_kc, uint8_t *P,
                         int64_t ldp, hipStream_t s, int64_t kfill) {
  if (kfill < k) kfill = k;
  if (kfill == 0 || n == 0) return hipSuccess;
  if (b_kc) {
    int64_t blocks = ((kfill + 15) / 16 * n + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(pack_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, k, kfill, n, B, ldb,
                       P, ldp, (int)aligned16(B, ldb), (int)aligned16(P, ldp));
  } else {
    const int64_t tiles_k = (kfill + PT - 1) / PT, tiles_n = (n + PT - 1) / PT;
    if (tiles_k * tiles_n > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_transpose_kernel, dim3((unsigned)(tiles_k * tiles_n)), dim3(256), 0, s,
                       k, kfill, n, B, ldb, P, ldp, (int)aligned16(B, ldb), (int)aligned16(P, ldp),
                       (int)tiles_n);
  }
  return hipGetLastError();
}

}  // namespace mip
