// Instantiation of the direct-to-LDS tile kernel for 64 x 128 workgroup tiles.
#include "dma_tile.h"

namespace mip {

bool dma_eligible_64x128(const Problem &p) { return dma_tile_eligible_for<64, 128>(p); }

hipError_t launch_dma_64x128(const Problem &p, int splits, hipStream_t s) {
  return launch_dma_tile_for<64, 128>(p, splits, s);
}

}  // namespace mip
