// RMSNorm instantiations of the restoration kernel, and the launch-shape selection shared by
// all variants.
#include "restore_kernel.inc"

namespace hc {

hipError_t launch_mode0(const RestoreArgs& a, const TileGrid& g, unsigned grid, const LayerBatch* mb,
                        hipStream_t stream) {
  return launch_mode<0>(a, g, grid, mb, stream);
}
hipError_t configure_mode0() { return configure_mode<0>(); }

hipError_t configure_kernels() {
  hipError_t e = configure_mode0();
  if (e != hipSuccess) return e;
  e = configure_mode1();
  if (e != hipSuccess) return e;
  return configure_mode2();
}

hipError_t launch_restore(const RestoreArgs& a, LayerBatch* batch, int n_layers, hipStream_t stream) {
  if (a.n_tok <= 0) return hipSuccess;
  TileGrid g;
  const int slots = choose_tile_grid(2 * a.d_kv_pad / kTileF, (a.n_tok + kTileT - 1) / kTileT, g);
  unsigned grid = (unsigned)slots;
  if (batch) {
    batch->slots_per_layer = (int32_t)grid;
    grid *= (unsigned)n_layers;
  }
  if (a.mode == 0) return launch_mode0(a, g, grid, batch, stream);
  if (a.mode == 1) return launch_mode1(a, g, grid, batch, stream);
  return launch_mode2(a, g, grid, batch, stream);
}

}  // namespace hc
