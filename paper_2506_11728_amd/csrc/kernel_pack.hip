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
// One packing job: the k x n matrix at B (k_contiguous: column j at B + j * ldb; else row
// p at B + p * ldb) to P, column j at P + j * ldp, entries k .. kfill - 1 of every packed
// column written as zeros (kfill == k: none).
struct PackJob {
  int64_t k, kfill, n;
  const uint8_t *B;
  int64_t ldb;
  uint8_t *P;
  int64_t ldp;
  int k_contiguous, wide_load, wide_store;
  int tiles_n;      // transposing job: 64 x 64 tiles along n
  unsigned blocks;  // workgroups this job is given
};

// block: this workgroup's number within the job
__device__ __forceinline__ void pack_transpose_body(const PackJob &J, unsigned block, uint8_t *tile) {
  const int64_t k = J.k, kfill = J.kfill, n = J.n, ldb = J.ldb, ldp = J.ldp;
  const uint8_t *B = J.B;
  uint8_t *P = J.P;
  const int wide_load = J.wide_load, wide_store = J.wide_store, tiles_n = J.tiles_n;
  const int t = threadIdx.x;
  const int64_t p0 = (int64_t)(block / tiles_n) * PT, n0 = (int64_t)(block % tiles_n) * PT;
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
__device__ __forceinline__ void pack_copy_body(const PackJob &J, unsigned block) {
  const int64_t k = J.k, kfill = J.kfill, n = J.n, ldb = J.ldb, ldp = J.ldp;
  const uint8_t *B = J.B;
  uint8_t *P = J.P;
  const int wide_load = J.wide_load, wide_store = J.wide_store;
  const int64_t pieces = (kfill + 15) / 16;
  const int64_t total = pieces * n;
  for (int64_t i = (int64_t)block * 256 + threadIdx.x; i < total; i += (int64_t)J.blocks * 256) {
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

// One or two jobs in one launch: the first a.blocks workgroups work on a, the rest on b
// (Pack A and Pack B of a GEMM are independent of each other).
__global__ __launch_bounds__(256) void pack_kernel(PackJob a, PackJob b) {
  __shared__ __attribute__((aligned(16))) uint8_t tile[PT * PITCH];
  const bool first = blockIdx.x < a.blocks;  // workgroup-uniform
  const PackJob &J = first ? a : b;
  const unsigned block = first ? blockIdx.x : blockIdx.x - a.blocks;
  if (J.k_contiguous) pack_copy_body(J, block);
  else pack_transpose_body(J, block, tile);
}

bool aligned16(const void *p, int64_t ld) {
  return reinterpret_cast<uintptr_t>(p) % 16 == 0 && ld % 16 == 0;
}

// false: the job is too large for one launch
bool make_job(int64_t k, int64_t kfill, int64_t n, const uint8_t *B, int64_t ldb, bool b_kc,
              uint8_t *P, int64_t ldp, PackJob *out) {
  PackJob J;
  J.k = k; J.kfill = kfill < k ? k : kfill; J.n = n;
  J.B = B; J.ldb = ldb; J.P = P; J.ldp = ldp;
  J.k_contiguous = b_kc;
  J.wide_load = aligned16(B, ldb);
  J.wide_store = aligned16(P, ldp);
  J.tiles_n = 1;
  if (J.kfill == 0 || n == 0) {
    J.blocks = 0;
  } else if (b_kc) {
    int64_t blocks = ((J.kfill + 15) / 16 * n + 255) / 256;
    J.blocks = (unsigned)(blocks > 256 * 64 ? 256 * 64 : blocks);
  } else {
    const int64_t tiles_k = (J.kfill + PT - 1) / PT, tiles_n = (n + PT - 1) / PT;
    if (tiles_k * tiles_n > 0x3fffffff) return false;
    J.tiles_n = (int)tiles_n;
    J.blocks = (unsigned)(tiles_k * tiles_n);
  }
  *out = J;
  return true;
}

// One wave per column of a k-contiguous matrix: the sum of its k bytes read as signed 8-bit
// values.  WIDE: k a multiple of 16 and every column 16-byte aligned.
template <bool WIDE>
__global__ __launch_bounds__(256) void column_sums_kernel(const uint8_t *P, int64_t ldp, int64_t k,
                                                          int64_t n, int32_t *sums) {
  const int lane = threadIdx.x & 63;
  const int64_t col = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (col >= n) return;
  int sum = 0;
  if (WIDE) {
    const v4i_pack *src = reinterpret_cast<const v4i_pack *>(P + col * ldp);
    for (int64_t c = lane; c < k / 16; c += 64) {
      const v4i_pack v = src[c];
#pragma unroll
      for (int e = 0; e < 4; ++e) sum = __builtin_amdgcn_sdot4(v[e], 0x01010101, sum, false);
    }
  } else {
    const int8_t *src = reinterpret_cast<const int8_t *>(P + col * ldp);
    for (int64_t c = lane; c < k; c += 64) sum += src[c];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) sums[col] = sum;
}

}  // namespace

hipError_t launch_column_sums(int64_t k, int64_t n, const uint8_t *P, int64_t ldp, int32_t *sums,
                              hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if ((n + 3) / 4 > 0x7fffffff) return hipErrorInvalidValue;
  const bool wide = k % 16 == 0 && ldp % 16 == 0 && reinterpret_cast<uintptr_t>(P) % 16 == 0;
  const dim3 grid((unsigned)((n + 3) / 4));
  if (wide) hipLaunchKernelGGL(column_sums_kernel<true>, grid, dim3(256), 0, s, P, ldp, k, n, sums);
  else hipLaunchKernelGGL(column_sums_kernel<false>, grid, dim3(256), 0, s, P, ldp, k, n, sums);
  return hipGetLastError();
}

hipError_t launch_pack_b(int64_t k, int64_t n, const uint8_t *B, int64_t ldb, bool b_kc, uint8_t *P,
                         int64_t ldp, hipStream_t s, int64_t kfill) {
  PackJob J, none = {};
  if (!make_job(k, kfill, n, B, ldb, b_kc, P, ldp, &J)) return hipErrorInvalidValue;
  if (J.blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(pack_kernel, dim3(J.blocks), dim3(256), 0, s, J, none);
  return hipGetLastError();
}

hipError_t launch_pack_pair(int64_t k, int64_t kfill, int64_t m, const uint8_t *A, int64_t lda,
                            bool a_kc, uint8_t *Ap, int64_t n, const uint8_t *B, int64_t ldb,
                            bool b_kc, uint8_t *Bp, int64_t ldp, hipStream_t s) {
  PackJob a, b;
  if (!make_job(k, kfill, m, A, lda, a_kc, Ap, ldp, &a) || !make_job(k, kfill, n, B, ldb, b_kc, Bp, ldp, &b))
    return hipErrorInvalidValue;
  if (a.blocks + b.blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(pack_kernel, dim3(a.blocks + b.blocks), dim3(256), 0, s, a, b);
  return hipGetLastError();
}

}  // namespace mip
