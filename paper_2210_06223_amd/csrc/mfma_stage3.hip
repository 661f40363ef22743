// Matrix-core instantiations of the fused sparse bottleneck: ResNet-101 stage 3 (14x14x1024, mid 256).
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {
//             C     M   S PPW R1MAX NW KC NSTG conv1  conv2 RD2  conv3 NB3 RD3
// Weights are 2.2 MB: one 8-wave workgroup per CU whose batch is as large as LDS allows -- up to 32 patches at
// S=2 (128 output rows; what bounds it in practice is the 160 y1 rows of distinct window pixels), two tiles at
// S=7 (side by side they share a window column: 144 rows) -- so that the weights stream through a CU once
// for everything the CU has to do, up to an activation ratio of 1 at batch 128.
// (weight rings of 4 and 2 steps: deeper ones measured the same)
using K_s3 = Cfg<1024, 256, 2, 32, 160, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;    // S=2
using K_s3s7 = Cfg<1024, 256, 7, 2, 144, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;   // S=7 (also the dense tile)
using K_s3s1 = Cfg<1024, 256, 1, 64, 160, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;  // S=1 (pixel level)
}  // namespace

#define LASNET_CFGS(X) X(K_s3) X(K_s3s7) X(K_s3s1)
LASNET_DEFINE_VARIANT_TABLE(stage3, LASNET_CFGS)
}  // namespace lasnet
