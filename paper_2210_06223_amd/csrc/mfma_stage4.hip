// Matrix-core instantiations of the fused sparse bottleneck: ResNet-101 stage 4 (7x7x2048, mid 512).
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {
//             C     M   S PPW R1MAX NW KC NSTG conv1  conv2 RD2  conv3 NB3 RD3
// 8.9 MB of weights on 7x7 maps: a workgroup is bound by streaming the weights whatever it
// computes, so it takes up to 16 pixel-level patches and their 3x3 neighbourhoods.
using K_s4 = Cfg<2048, 512, 1, 16, 96, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;     // S=1
}  // namespace

#define LASNET_CFGS(X) X(K_s4)
LASNET_DEFINE_VARIANT_TABLE(stage4, LASNET_CFGS)
}  // namespace lasnet
