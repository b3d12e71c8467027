// Instantiation of the direct-to-LDS tile kernel for 128 x 64 workgroup tiles.
#include "dma_tile.h"

namespace mip {

bool dma_eligible_128x64(const Problem &p) { return dma_tile_eligible_for<128, 64>(p); }

hipError_t launch_dma_128x64(const Problem &p, int splits, hipStream_t s) {
  return launch_dma_tile_for<128, 64>(p, splits, s);
}

}  // namespace mip
