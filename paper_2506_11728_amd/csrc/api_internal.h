// Shared between the files of the C-ABI layer.  Not installed.
#pragma once
#include "../../include/mipgemm.h"
#include "mip_internal.h"

namespace mip {

inline bool order_ok(int o) { return o == MIPGEMM_ROW_MAJOR || o == MIPGEMM_COL_MAJOR; }

// a strided batch of problems of one shape (count 1: a single problem)
struct Batch {
  int64_t count = 1;
  int64_t stride_a = 0, stride_b = 0, stride_c = 0;  // elements between consecutive problems
};

// Fills `out` and returns 0, or returns the negative argument number (numbered as in the
// single-problem GEMM entry points).
int validate_and_normalise(int a_unsigned, int b_unsigned, int64_t m, int64_t n, int64_t k,
                           const void *A, int64_t lda, int orderA, const void *B, int64_t ldb,
                           int orderB, void *C, int64_t ldc, int orderC, int mode,
                           void *workspace, size_t workspace_bytes, Problem *out);

// Bytes of workspace with which this call would take the packed route (operands that the
// direct-to-LDS kernels cannot stream, and a product large enough for packing to pay), else 0.
size_t packed_route_bytes(const Problem &p);

// Enqueues the kernels of a plan.
hipError_t launch_plan(const Problem &p, const Plan &plan, hipStream_t s);

// Validates, plans and launches one GEMM call.  out_float: C holds floats and receives
// float(sum) * scale (the f32 entry points).
int run_gemm(int a_unsigned, int b_unsigned, int out_float, float scale, int64_t m, int64_t n,
             int64_t k, const void *A, int64_t lda, int orderA, const void *B, int64_t ldb,
             int orderB, void *C, int64_t ldc, int orderC, int mode, void *workspace,
             size_t workspace_bytes, void *stream, const Batch &batch = Batch(),
             const int32_t *ksum = nullptr);  // ksum: see Problem::ksum (pre-packed weights)

}  // namespace mip
