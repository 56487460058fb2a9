// Persistent weights-resident instances: single NHWC convolutions with small weights, and
// back-to-back convolutions (RF-resident fusion).
#include "instances.hpp"
namespace bolt {
#define SC(BM, BK, NW, N0T, NS) BOLT_STREAM_FPROP_INSTANCE(BM, BK, NW, N0T, NS, 1, 0)
#define SB(BM, BK, NW, N0T, N1T, NS) BOLT_STREAM_INSTANCE(BM, BK, NW, N0T, N1T, NS, 1, 0)
void register_conv_stream_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {
      SC(256, 64, 4, 64, 2),  SC(128, 64, 4, 64, 4),  SC(256, 64, 8, 64, 3),  SC(128, 64, 4, 128, 3),
      SC(256, 64, 4, 128, 2), SC(128, 64, 4, 256, 3), SC(256, 64, 8, 256, 2),
  };
  for (const auto& t : table) v.push_back(t);
}
void register_b2b_conv_stream_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      SB(128, 64, 4, 64, 256, 2), SB(128, 32, 4, 64, 256, 4), SB(64, 64, 2, 64, 256, 4), SB(128, 64, 4, 64, 64, 3),
      SB(256, 64, 8, 64, 64, 2),  SB(128, 64, 4, 64, 128, 3), SB(128, 64, 4, 128, 128, 2),
  };
  for (const auto& t : table) v.push_back(t);
}
#define BD(BM, BK, NW, N0T, N1T, NS) BOLT_B2B_DMA_INSTANCE(BM, BK, NW, N0T, N1T, NS, 1)
void register_b2b_conv_dma_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      BD(128, 64, 4, 64, 256, 2), BD(128, 64, 4, 64, 256, 3), BD(64, 64, 2, 64, 256, 3), BD(256, 64, 8, 64, 256, 2),
      BD(128, 64, 4, 64, 64, 3),  BD(128, 64, 4, 64, 128, 3), BD(128, 64, 4, 128, 128, 2), BD(64, 64, 2, 32, 32, 3),
      BD(128, 64, 4, 64, 64, 2),  BD(256, 64, 8, 64, 64, 2),  BD(256, 64, 8, 64, 64, 3),   BD(128, 32, 4, 64, 64, 4),
      BD(128, 32, 4, 64, 64, 3),  BD(64, 64, 2, 64, 64, 3),   BD(256, 64, 4, 64, 64, 2),   BD(256, 32, 4, 64, 64, 3),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
