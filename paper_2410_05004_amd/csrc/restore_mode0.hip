// RMSNorm instantiations of the restoration kernel, and the launch-shape selection shared by
// all variants.
#include "restore_kernel.inc"

namespace hc {

hipError_t launch_mode0(const RestoreArgs& a, const TileGrid& g, unsigned grid, const LayerBatch* mb,
                        const SplitPlan* sp, hipStream_t stream) {
  return launch_mode<0>(a, g, grid, mb, sp, stream);
}
hipError_t configure_mode0() { return configure_mode<0>(); }

hipError_t configure_kernels() {
  hipError_t e = configure_mode0();
  if (e != hipSuccess) return e;
  e = configure_mode1();
  if (e != hipSuccess) return e;
  return configure_mode2();
}

bool restore_would_split(const RestoreArgs& a, SplitPlan& sp, TileGrid& g_main) {
  if (!a.split_ws || a.n_tok <= 0) return false;
  return plan_split(2 * a.d_kv_pad / kTileF, (a.n_tok + kTileT - 1) / kTileT, a.d_model / (2 * kTileK), a.split_force != 0, sp, g_main);
}

hipError_t launch_restore(const RestoreArgs& a, LayerBatch* batch, int n_layers, hipStream_t stream) {
  if (a.n_tok <= 0) return hipSuccess;
  TileGrid g;
  SplitPlan sp;
  const SplitPlan* use_split = nullptr;
  unsigned grid = 0;
  if (!batch && restore_would_split(a, sp, g)) {
    sp.ws = a.split_ws;
    use_split = &sp;
  } else {
    grid = (unsigned)choose_tile_grid(2 * a.d_kv_pad / kTileF, (a.n_tok + kTileT - 1) / kTileT, g);
    if (batch) {
      batch->slots_per_layer = (int32_t)grid;
      grid *= (unsigned)n_layers;
    }
  }
  if (a.mode == 0) return launch_mode0(a, g, grid, batch, use_split, stream);
  if (a.mode == 1) return launch_mode1(a, g, grid, batch, use_split, stream);
  return launch_mode2(a, g, grid, batch, use_split, stream);
}

}  // namespace hc
