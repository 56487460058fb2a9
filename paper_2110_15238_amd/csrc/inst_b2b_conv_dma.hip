// Multi-stage fused convolution pairs (3x3 -> 1x1, RF-resident fusion) with direct-to-LDS operand loads.
#include "instances.hpp"
namespace bolt {
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
