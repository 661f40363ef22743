// Matrix-core instantiations of the fused sparse bottleneck: ResNet-101 stage 1 (56x56x256, mid 64).
#include "bottleneck_mfma.hpp"
#include "bottleneck_stream.hpp"

namespace lasnet {
namespace {
//             C     M   S PPW R1MAX NW KC NSTG conv1  conv2 RD2  conv3 NB3 RD3
// Two 4-wave workgroups per CU (see stage 2); x is only 4 chunks of 64 channels deep, so all of a
// batch's x is requested at once (NSTG = 4).
using K_s1 = Cfg<256, 64, 8, 1, 112, 4, 64, 4, 1, 4, 1, 4, 6, 1, 4, 4, 2>;       // S=8
using K_s1s4 = Cfg<256, 64, 4, 4, 112, 4, 64, 4, 1, 4, 1, 4, 6, 1, 4, 4, 2>;     // S=4 (the block of Table 1)
using K_s1s7 = Cfg<256, 64, 7, 1, 96, 4, 64, 4, 1, 4, 1, 4, 6, 1, 4, 4, 2>;      // S=7 (dense tile)
using K_s1s2 = Cfg<256, 64, 2, 8, 112, 4, 64, 4, 1, 4, 1, 4, 6, 1, 4, 4, 2>;     // S=2
using K_s1s1 = Cfg<256, 64, 1, 16, 112, 4, 64, 4, 1, 4, 1, 4, 6, 1, 4, 4, 2>;    // S=1 (pixel level)
}  // namespace

// S=8 runs on the streaming, weight-stationary kernel; it reads the buffer that K_s1's packing
// writes (K_s1 is instantiated for its packing only).  Maps beyond the kernel's 32-bit byte offsets
// are left to the generic kernel by the dispatcher.
using KS_s1 = StreamCfg<256, 64, 8>;

#define LASNET_CFGS(X) X(K_s1s4) X(K_s1s7) X(K_s1s2) X(K_s1s1)
const MfmaVariant* mfma_variants_stage1(int* n) {
  static const MfmaVariant table[] = {
      MfmaVariant{K_s1::C, K_s1::M, K_s1::S, K_s1::PACKED_ELEMS * 2, stream_max_map_bytes<KS_s1>(),
                  &prepare_stream<KS_s1>, &pack_one<K_s1>, &launch_stream<KS_s1>},
      LASNET_CFGS(LASNET_VARIANT_ENTRY)};
  *n = (int)(sizeof(table) / sizeof(table[0]));
  return table;
}
}  // namespace lasnet
