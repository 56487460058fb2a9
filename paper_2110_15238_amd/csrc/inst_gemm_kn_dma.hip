// GEMM instances, B stored row-major [K][N], direct-to-LDS pipeline with transposing LDS reads.
#include "instances.hpp"
namespace bolt {
void register_gemm_kn_dma_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {BOLT_FPROP_DMA_KN_TILE_LIST(BOLT_FPROP_DMA_KN_INSTANCE), BOLT_FPROP_PP_KN_INSTANCE(16, 64, 256),
                                        BOLT_FPROP_PP_KN_INSTANCE(16, 64, 224)};
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
