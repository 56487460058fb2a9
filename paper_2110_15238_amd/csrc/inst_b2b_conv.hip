// Back-to-back convolution instances: NHWC activations, KRSC weights.
#include "instances.hpp"
namespace bolt {
#define RF(BM, BK, NW, N0T, N1T) BOLT_B2B_RF_INSTANCE(BM, BK, NW, N0T, N1T, 1, 0)
#define LD(BM, BK, A, B, C, D, N0T, N1T) BOLT_B2B_LDS_INSTANCE(BM, BK, A, B, C, D, N0T, N1T, 1, 0)
void register_b2b_conv_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      RF(128, 64, 4, 64, 256), RF(128, 64, 4, 64, 64),
      RF(256, 64, 4, 64, 64),  RF(128, 64, 4, 64, 128), RF(128, 64, 4, 32, 32),  RF(128, 64, 4, 128, 128),
      LD(128, 64, 4, 1, 2, 2, 64, 256), LD(128, 64, 4, 1, 1, 4, 64, 256), LD(128, 64, 4, 1, 2, 2, 64, 64),
      LD(64, 64, 2, 2, 2, 2, 64, 64),   LD(128, 64, 2, 2, 2, 2, 128, 128), LD(64, 64, 2, 1, 2, 1, 32, 32),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
