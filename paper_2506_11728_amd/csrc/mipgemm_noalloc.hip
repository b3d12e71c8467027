// GEMM entry point for callers that cannot allocate device memory and have no workspace
// to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc.  It is mipgemm_s8s8s32 with the packed route's buffers (Pack A / Pack B of the
// paper's Section 4.1: aligned, k-contiguous, zero-padded copies of operands that cannot be
// streamed as they are stored) in a static device array instead of a caller's workspace.
#include <mutex>

#include "api_internal.h"

namespace {

constexpr size_t SCRATCH_BYTES = MIPGEMM_STATIC_SCRATCH_BYTES;

// One copy per GPU the library runs on, held until the process ends.  The name is a host-side
// stand-in only: host code uses the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
struct PerDevice {
  std::once_flag once;
  void *ptr = nullptr;
  hipError_t status = hipErrorNotInitialized;
};
PerDevice g_device[MAX_DEVICES];

// The array's address on the current device, looked up once per device with that device current.
hipError_t scratch_on_current_device(void **out) {
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
  PerDevice &d = g_device[device];
  std::call_once(d.once, [&d] {
    void *p = nullptr;
    d.status = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    d.ptr = d.status == hipSuccess ? p : nullptr;
  });
  if (d.status != hipSuccess) return d.status;
  *out = d.ptr;
  return hipSuccess;
}

}  // namespace

extern "C" {

size_t mipgemm_static_scratch_bytes(void) { return SCRATCH_BYTES; }

int mipgemm_s8s8s32_noalloc(int64_t m, int64_t n, int64_t k, const int8_t *A, int64_t lda, int orderA,
                            const int8_t *B, int64_t ldb, int orderB, int32_t *C, int64_t ldc,
                            int orderC, int mode, void *stream) {
  mip::Problem p;
  const int rc = mip::validate_and_normalise(0, 0, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc,
                                             orderC, mode, nullptr, 0, &p);
  if (rc != 0) return rc;
  const size_t need = mip::packed_route_bytes(p);
  if (need > SCRATCH_BYTES) return MIPGEMM_ERR_STATIC_SCRATCH;  // nothing enqueued, nothing touched
  void *ptr = nullptr;
  if (need > 0) {
    const hipError_t e = scratch_on_current_device(&ptr);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  // with need == 0 the call runs on the kernels that read the operands in place
  return mip::run_gemm(0, 0, 0, 1.0f, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                       ptr, need > 0 ? SCRATCH_BYTES : 0, stream);
}

}  // extern "C"
