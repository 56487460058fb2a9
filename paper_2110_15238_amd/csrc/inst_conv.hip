// Implicit-GEMM NHWC convolution instances (weights KRSC).
#include "instances.hpp"
namespace bolt {
void register_conv_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {BOLT_FPROP_DMA_TILE_LIST(BOLT_FPROP_DMA_INSTANCE, 1),
                                        BOLT_FPROP_DMA_KG_TILE_LIST(BOLT_FPROP_DMA_KG_INSTANCE, 1),
                                        BOLT_FPROP_DMA_1STAGE_TILE_LIST(BOLT_FPROP_DMA_INSTANCE, 1),
                                        BOLT_FPROP_PP_INSTANCE(1, 16, 64, 256),
                                        BOLT_FPROP_PP_INSTANCE(1, 16, 64, 224)};
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
