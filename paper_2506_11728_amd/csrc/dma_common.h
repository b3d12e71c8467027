// Helpers shared by the kernels that stream operands global -> LDS directly.
#pragma once
#include <type_traits>

#include "epilogue.h"
#include "lds_layout.h"
#include "mip_internal.h"

namespace mip {

// One wave-wide direct load: lane l's 16 bytes from sbase + voff land in LDS at
// lds_addr + 16 * l.  Written as inline assembly so that the compiler's
// automatic wait-count insertion, which would drain every outstanding load
// before any LDS read, stays out of the pipeline; the kernel places its own
// s_waitcnt vmcnt before the barrier that publishes a stage.  M0 carries the
// LDS base and needs one wait state before the load reads it.  M0 is reserved
// in this compiler: the register allocator never holds a value in it, and naming
// it on the clobber list only draws a "reserved register" warning.  The compiler
// sets M0 itself, right before use, for dynamically indexed register arrays and
// message sends; the kernels that call this keep every register array fully
// unrolled and send no messages, so nothing of the compiler's lives in M0 here.
__device__ __forceinline__ void dma16(uint32_t voff, const uint8_t *sbase, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(sbase), "s"(lds_addr)
      :);
}

// The same with a full 64-bit address per lane (lanes may point anywhere).
__device__ __forceinline__ void dma16_at(const uint8_t *addr, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off"
      :
      : "v"(addr), "s"(lds_addr)
      :);
}

// "my loads of the next block have landed (N newer loads may still fly), my LDS
// reads are complete; meet the other waves": after this the next stage is
// visible to the whole workgroup and the stage read two steps ago may be refilled.
template <int N>
__device__ __forceinline__ void publish_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const uint8_t *p) {
  return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const uint8_t *)p);
}

// Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of
// them, each with its own L2), so every XCD gets a contiguous run of tiles, and
// the tiles are walked in groups of 8 tile-rows so that the workgroups resident
// on one XCD share A row-panels and B column-panels.  Returns false for the
// padding workgroups at the end of the grid.
__device__ __forceinline__ bool tile_of_workgroup(int tiles_m, int tiles_n, int *tm, int *tn) {
  const int ntiles = tiles_m * tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  const int lid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (blockIdx.x / 8 >= per_xcd || lid >= ntiles) return false;
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int first_m = (lid / per_group) * GROUP;
  const int gsz = tiles_m - first_m < GROUP ? tiles_m - first_m : GROUP;
  *tm = first_m + (lid % per_group) % gsz;
  *tn = (lid % per_group) / gsz;
  return true;
}

}  // namespace mip
