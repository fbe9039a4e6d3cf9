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
  g.nf = 2 * a.d_kv_pad / kTileF;
  g.nt = (a.n_tok + kTileT - 1) / kTileT;
  // Super-tile shape: fewest rounds on the busiest XCD (an XCD runs 32 workgroups at a
  // time, one per CU), then the most row sharing (smallest 1/GF + 1/GT), then fewest slots.
  // Of two shapes that tie (GF x GT = 4 x 8 and 8 x 4 for 8 x 32 tiles) the one with fewer
  // feature tiles is met first and kept: it measured 105.4 against 107.0 us per layer.
  int best_rounds = 1 << 30, best_slots = 1 << 30, best_share = 1 << 30;
  g.gf_shift = g.g_shift = 0;
  for (int fs = 0; fs <= 5; ++fs) {
    for (int ts = 0; fs + ts <= 5; ++ts) {
      const int gf = 1 << fs, gt = 1 << ts;
      const int n_super = ((g.nf + gf - 1) / gf) * ((g.nt + gt - 1) / gt);
      const int slots = (n_super + 7) / 8 * gf * gt;      // workgroup slots per XCD
      const int rounds = (slots + 31) / 32;
      const int share = (32 >> fs) + (32 >> ts);          // 32 * (1/GF + 1/GT)
      if (rounds < best_rounds || (rounds == best_rounds && share < best_share) ||
          (rounds == best_rounds && share == best_share && slots < best_slots)) {
        best_rounds = rounds; best_share = share; best_slots = slots;
        g.gf_shift = fs; g.g_shift = fs + ts;
      }
    }
  }
  g.nsf = (g.nf + (1 << g.gf_shift) - 1) >> g.gf_shift;
  unsigned grid = (unsigned)best_slots * 8u;
  if (batch) {
    batch->slots_per_layer = (int32_t)grid;
    grid *= (unsigned)n_layers;
  }
  if (a.mode == 0) return launch_mode0(a, g, grid, batch, stream);
  if (a.mode == 1) return launch_mode1(a, g, grid, batch, stream);
  return launch_mode2(a, g, grid, batch, stream);
}

}  // namespace hc
