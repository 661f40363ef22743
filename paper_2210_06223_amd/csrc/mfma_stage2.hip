// Matrix-core instantiations of the fused sparse bottleneck: ResNet-101 stage 2 (28x28x512, mid 128).
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {
//             C     M   S PPW R1MAX NW KC NSTG conv1  conv2 RD2  conv3 NB3 RD3
// Stages 1 and 2 have small weights (0.14 / 0.56 MB) and large maps: two 4-wave workgroups per
// CU (<= 80 KB of LDS each), so that one workgroup's HBM-bound conv1 overlaps the other's
// matrix work, instead of one 8-wave workgroup whose phases leave HBM or the matrix cores idle.
using K_s2 = Cfg<512, 128, 4, 4, 112, 4, 64, 3, 1, 4, 1, 4, 4, 1, 4, 4, 2>;      // S=4
using K_s2s7 = Cfg<512, 128, 7, 1, 96, 4, 64, 4, 1, 4, 1, 4, 4, 1, 4, 4, 2>;     // S=7 (dense tile)
using K_s2s2 = Cfg<512, 128, 2, 8, 112, 4, 64, 3, 1, 4, 1, 4, 4, 1, 4, 4, 2>;    // S=2
using K_s2s1 = Cfg<512, 128, 1, 24, 112, 4, 64, 3, 1, 4, 1, 4, 4, 1, 4, 4, 2>;   // S=1 (pixel level)
}  // namespace

#define LASNET_CFGS(X) X(K_s2) X(K_s2s7) X(K_s2s2) X(K_s2s1)
LASNET_DEFINE_VARIANT_TABLE(stage2, LASNET_CFGS)
}  // namespace lasnet
