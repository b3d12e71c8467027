// The counters of split k through partial-sum slots (combine_k_ranges in epilogue.h): one
// 32-bit ticket counter per tile, zero whenever no call is using it.  They live in a static
// device array, zero from the moment the code object is loaded, because a caller's workspace
// arrives with unknown contents and zeroing it would cost the very launch this scheme saves.
// Every call takes the next `count` counters of the ring, so calls in flight at the same
// time (other streams, other threads, other nodes of a captured graph) work on different
// counters; a range is handed out again only after the whole ring has gone round.
#include <atomic>
#include <mutex>

#include "mip_internal.h"

namespace mip {

namespace {

constexpr int64_t TICKETS = 1 << 20;  // 4 MiB per device
static __device__ unsigned g_tickets[TICKETS];

constexpr int MAX_DEVICES = 64;
struct PerDevice {
  std::once_flag once;
  unsigned *base = nullptr;
  hipError_t status = hipErrorNotInitialized;
  std::atomic<uint64_t> cursor{0};
};
PerDevice g_device[MAX_DEVICES];

}  // namespace

hipError_t splitk_tickets(int64_t count, unsigned **out) {
  if (count < 1 || count > TICKETS / 4) return hipErrorInvalidValue;  // the caller falls back to atomics
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
  PerDevice &d = g_device[device];
  std::call_once(d.once, [&d] {
    void *p = nullptr;
    d.status = hipGetSymbolAddress(&p, HIP_SYMBOL(g_tickets));
    d.base = d.status == hipSuccess ? static_cast<unsigned *>(p) : nullptr;
  });
  if (d.status != hipSuccess) return d.status;
  // the next `count` counters that do not straddle the end of the ring
  uint64_t at = d.cursor.load(std::memory_order_relaxed), first;
  do {
    first = at + (uint64_t)count > (uint64_t)TICKETS ? 0 : at;
  } while (!d.cursor.compare_exchange_weak(at, first + (uint64_t)count, std::memory_order_relaxed));
  *out = d.base + first;
  return hipSuccess;
}

}  // namespace mip
