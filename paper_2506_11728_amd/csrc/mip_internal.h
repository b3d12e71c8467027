// Internal interface between the C-ABI layer and the HIP kernels.  Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mip {

// The problem after the host has normalised it: C is always row-major here (a
// column-major C is the row-major C^T = B^T A^T, so the host swaps the operand
// roles and flips their orders; paper Section 3, closing paragraph), and each
// 8-bit operand is described by two element strides, one of which is 1.
struct Problem {
  int64_t m, n, k;
  const void *A;  // A(i,p) at A[i*a_sm + p*a_sk]
  int64_t a_sm, a_sk;
  const void *B;  // B(p,j) at B[p*b_sk + j*b_sn]
  int64_t b_sk, b_sn;
  int32_t *C;  // C(i,j) at C[i*ldc + j]
  int64_t ldc;
  int a_unsigned, b_unsigned;
  int accumulate;
};

enum Variant {
  VARIANT_NONE = 0,   // nothing to launch (m == 0 or n == 0, or k == 0 with accumulate)
  VARIANT_FILL,       // k == 0, overwrite: C := 0
  VARIANT_SIMPLE,     // one thread per C element, any layout
  VARIANT_DMA256,     // MFMA, 256 x 256 tile, global->LDS direct loads, aligned full tiles only
  VARIANT_DMA256K128, // same, k blocks of 128 in two LDS stages
  VARIANT_TILE256,    // MFMA, 256 x 256 workgroup tile
  VARIANT_TILE128,    // MFMA, 128 x 128 workgroup tile
  VARIANT_TILE64,     // MFMA, 64 x 64 workgroup tile
  VARIANT_TILE64X256, // MFMA, 64 x 256 tile: few rows, many columns
  VARIANT_TILE256X64, // MFMA, 256 x 64 tile: many rows, few columns
  VARIANT_COUNT
};

const char *variant_name(Variant v);
// Kernel and, for the tile kernels, the number of k ranges worked on by separate
// workgroups (1 = no split).
struct Plan {
  Variant variant;
  int splits;
};
Plan choose_plan(const Problem &p);

hipError_t launch_fill_zero(const Problem &p, hipStream_t s);
hipError_t launch_simple(const Problem &p, hipStream_t s);
hipError_t launch_tile(const Problem &p, Variant v, int splits, hipStream_t s);
bool dma_eligible(const Problem &p, bool deep);  // deep: k blocks of 128 instead of 64
hipError_t launch_dma(const Problem &p, bool deep, hipStream_t s);

}  // namespace mip
