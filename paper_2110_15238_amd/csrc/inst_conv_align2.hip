// Alignment-2 convolution instances: input channel counts that are even but not multiples of 8.
// These are what an unpadded layer has to run on; Table 3 measures channel padding against them.
#include "instances.hpp"
namespace bolt {
#define A2(BM, BN, BK, WM, WN) BOLT_FPROP_INSTANCE(BM, BN, BK, WM, WN, 2, 2)
void register_conv_align2_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {
      A2(64, 32, 64, 2, 1), A2(128, 32, 64, 4, 1), A2(64, 64, 64, 2, 2),   A2(128, 64, 64, 4, 1),
      A2(32, 64, 64, 1, 2), A2(256, 64, 32, 4, 2), A2(128, 128, 32, 2, 2),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
