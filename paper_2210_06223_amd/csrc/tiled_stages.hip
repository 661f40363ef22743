// Instantiations of the tiled schedule (conv1 | gather + conv3x3 | conv3 + scatter-add as three
// kernels): the two deep ResNet-101 stages, whose weights are too large for the fused kernel to
// stream through every CU.
#include "bottleneck_tiled.hpp"

namespace lasnet {
namespace {
//                   C     M  IMGS GPXMAX  slices of conv1 / conv2 / conv3
// 14x14x1024, mid 256: one image per group (196 pixels, 100 KB of y1 in LDS); conv1 keeps all 256
// output channels in one workgroup (x is read once), two tiles of 98 pixels per image.
using T_s3 = TiledCfg<1024, 256, 1, 196, 1, 2, 2>;
// 7x7x2048, mid 512: two images per group (98 pixels, 98 KB of y1 in LDS), four slices everywhere.
using T_s4 = TiledCfg<2048, 512, 2, 98, 4, 4, 4>;

template <class TC>
constexpr TiledVariant tiled_variant_of(bool preferred) {
  return TiledVariant{TC::C, TC::M, preferred, &tiled_takes<TC>, &tiled_workspace_bytes<TC>, &prepare_tiled<TC>,
                      &launch_tiled<TC>};
}
}  // namespace

// Which schedule wins was measured at batch 128 over activation rates 0.1 .. 1: at 7x7x2048 the tiled one
// at every rate (the fused kernel streams 8.9 MB of weights through every CU); at 14x14x1024 the fused
// one at every rate (three launches and their start-up latencies outweigh the saved weight traffic),
// so there the tiled schedule runs only on request.
const TiledVariant* tiled_variants(int* n) {
  static const TiledVariant table[] = {tiled_variant_of<T_s3>(false), tiled_variant_of<T_s4>(true)};
  *n = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
}  // namespace lasnet
