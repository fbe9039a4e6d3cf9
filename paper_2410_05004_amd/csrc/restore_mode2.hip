// LayerNorm + projection bias instantiations of the restoration kernel.
#include "restore_kernel.inc"

namespace hc {

hipError_t launch_mode2(const RestoreArgs& a, const TileGrid& g, unsigned grid, const LayerBatch* mb,
                        const SplitPlan* sp, hipStream_t stream) {
  return launch_mode<2>(a, g, grid, mb, sp, stream);
}
hipError_t configure_mode2() { return configure_mode<2>(); }

}  // namespace hc
