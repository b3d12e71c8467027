// Instantiation of the direct-to-LDS tile kernel for 256 x 64 workgroup tiles.
#include "dma_tile.h"

namespace mip {

bool dma_eligible_256x64(const Problem &p) { return dma_tile_eligible_for<256, 64>(p); }

hipError_t launch_dma_256x64(const Problem &p, int splits, hipStream_t s) {
  return launch_dma_tile_for<256, 64>(p, splits, s);
}

}  // namespace mip
