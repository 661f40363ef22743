// Matrix-core instantiations of the fused sparse bottleneck: ResNet-101 stage 3 (14x14x1024, mid 256).
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {
//             C     M   S PPW R1MAX NW KC NSTG conv1  conv2 RD2  conv3 NB3 RD3
// Weights are 2.2 MB: one 8-wave workgroup per CU with up to 16 patches (64 pixels at S=1), so that
// the weights stream through a CU once per batch.
// (weight rings of 4 and 2 steps: deeper ones cost registers, and spills inside the k-loops
// cost more than the extra latency cover is worth -- measured 46 us against 49)
using K_s3 = Cfg<1024, 256, 2, 16, 160, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;    // S=2
using K_s3s7 = Cfg<1024, 256, 7, 1, 96, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;    // S=7 (also the dense tile)
using K_s3s1 = Cfg<1024, 256, 1, 64, 160, 8, 64, 3, 1, 8, 1, 8, 4, 1, 8, 4, 2>;  // S=1 (pixel level)
}  // namespace

#define LASNET_CFGS(X) X(K_s3) X(K_s3s7) X(K_s3s1)
LASNET_DEFINE_VARIANT_TABLE(stage3, LASNET_CFGS)
}  // namespace lasnet
