// RMSNorm + projection bias instantiations of the restoration kernel.
#include "restore_kernel.inc"

namespace hc {

hipError_t launch_mode1(const RestoreArgs& a, const TileGrid& g, unsigned grid, const LayerBatch* mb,
                        const SplitPlan* sp, hipStream_t stream) {
  return launch_mode<1>(a, g, grid, mb, sp, stream);
}
hipError_t configure_mode1() { return configure_mode<1>(); }

}  // namespace hc
